"""The entry point that allocates nothing (excp_decompress_step_static) against the context's
excp_decompress_step, through the C ABI: two calls in a row, the second on a smaller tensor (the static
tables then still hold the first call's counts), then 16-bit weights, a blob written without
quantisation, an empty tensor and the refusals.  Outputs must be identical bit for bit; device memory
in use must not change across the calls."""
import numpy as np
import pytest
import torch

import paper_2406_11257_amd as X
from paper_2406_11257_amd import synth

pytestmark = pytest.mark.gpu


def make_case(n, seed, dtype=torch.float32):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    Wp = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0, 0.02, generator=g)
    step = torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-0.5, 0.5, generator=g)
    step = -1e-4 * torch.sign(step) * torch.log1p(-2.0 * step.abs().clamp_(max=0.49999997))
    W = Wp + step
    m = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0, 5e-5, generator=g)
    v = m * m * torch.empty(n, dtype=torch.float32, device="cuda").normal_(generator=g).exp_() + 1e-16
    return Wp.to(dtype), W.to(dtype), m, v


def compress(ctx, case, flags=0):
    n = case[0].numel()
    blob = torch.zeros(X.excp_blob_bound(n, 32 if flags & 4 else 4), dtype=torch.uint8, device="cuda")
    _, nbytes, st = ctx.excp_compress_step(*case, blob, synth.ALPHA, synth.BETA, 4, 5, flags=flags)
    return blob, nbytes, st


def both_ways(ctx, case, blob, nbytes):
    Wp = case[0]
    n = Wp.numel()
    ref = [torch.full((n,), 3.0, dtype=Wp.dtype, device="cuda")] + [torch.full((n,), 3.0, device="cuda") for _ in range(2)]
    got = [torch.full((n,), 5.0, dtype=Wp.dtype, device="cuda")] + [torch.full((n,), 5.0, device="cuda") for _ in range(2)]
    ctx.excp_decompress_step(Wp, blob, nbytes, *ref)
    X.excp_decompress_step_static(Wp, blob, nbytes, *got)
    for a, b in zip(got, ref):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    # weights only (the moment tables of the scratch array stay untouched by this call); the free device
    # memory the driver reports must be the same before and after
    w_only = torch.full((n,), 7.0, dtype=Wp.dtype, device="cuda")
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    X.excp_decompress_step_static(Wp, blob, nbytes, w_only, None, None)
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory in use changed across the call"
    assert torch.equal(w_only.view(torch.uint8), ref[0].view(torch.uint8))


def test_static_entry_point_equals_the_context_call_twice_in_a_row_second_smaller():
    ctx = X.Context(1 << 21)
    big = make_case(1_300_007, 1)           # 318 tiles, a ragged tail
    small = make_case(70_001, 2)            # 18 tiles: most of the static tables keep the first call's contents
    blob_b, nb_b, st_b = compress(ctx, big)
    blob_s, nb_s, st_s = compress(ctx, small)
    assert st_b.n_w > 0 and st_b.n_o > 0 and st_s.n_w > 0
    both_ways(ctx, big, blob_b, nb_b)
    both_ways(ctx, small, blob_s, nb_s)
    both_ways(ctx, big, blob_b, nb_b)       # and larger again
    # in place, as a chain of checkpoints would use it
    Wp = big[0].clone()
    expect = torch.empty_like(Wp)
    ctx.excp_decompress_step(big[0], blob_b, nb_b, expect, None, None)
    X.excp_decompress_step_static(Wp, blob_b, nb_b, Wp, None, None)
    assert torch.equal(Wp, expect)
    ctx.close()


def test_static_entry_point_other_blob_kinds_and_refusals():
    ctx = X.Context(1 << 20)
    for flags, dtype in ((X.EXCP_FLAG_W_F16, torch.float16), (X.EXCP_FLAG_W_BF16, torch.bfloat16),
                         (X.EXCP_FLAG_NO_QUANT, torch.float32), (X.EXCP_FLAG_NO_W2M, torch.float32)):
        case = make_case(300_017, 10 + flags, dtype)
        blob, nb, st = compress(ctx, case, flags)
        both_ways(ctx, case, blob, nb)
    # an empty tensor: header-only blob
    empty = tuple(torch.empty(0, dtype=torch.float32, device="cuda") for _ in range(4))
    blob, nb, _ = compress(ctx, empty)
    assert X.excp_decompress_step_static(empty[0], blob, nb, empty[1], None, None) == X.EXCP_OK
    # refusals: too large for the static tables (nothing is enqueued), wrong storage, a damaged blob
    case = make_case(5000, 3)
    blob, nb, _ = compress(ctx, case)
    L = X.lib()
    too_many = X.EXCP_STATIC_MAX_ELEMS + 1
    assert L.excp_decompress_step_static(0, None, case[0].data_ptr(), blob.data_ptr(), nb, too_many,
                                         None, None, None, 0) == X.EXCP_E_ARG
    assert L.excp_decompress_step_static(0, None, case[0].data_ptr(), blob.data_ptr(), nb, 5000,
                                         None, None, None, 0x30) == X.EXCP_E_ARG
    out = torch.empty(5000, dtype=torch.float16, device="cuda")
    assert X.excp_decompress_step_static(case[0].half(), blob, nb, out, None, None, check=False) == X.EXCP_E_BLOB
    bad = blob.clone(); bad[0] ^= 0xFF
    out = torch.empty(5000, device="cuda")
    assert X.excp_decompress_step_static(case[0], bad, nb, out, None, None, check=False) == X.EXCP_E_BLOB
    # and a good call afterwards still works
    both_ways(ctx, case, blob, nb)
    ctx.close()
