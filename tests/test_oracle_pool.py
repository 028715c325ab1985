"""The process pool that runs the oracle for the full-size GPU tests returns what a direct call of the
oracle returns (CPU only)."""
import hashlib

import numpy as np

import oracle as O
from oracle.pool import OraclePool, digest
from paper_2406_11257_amd import synth


def test_pool_results_equal_direct_calls():
    cfg = synth.config(0)
    params = dict(alpha=synth.ALPHA, beta=synth.BETA, nbits=4, iters=3)
    picks = (1, 5, 9, 11)
    cases = {f"t{i}": synth.draw_tensor(0, i, cfg.tensors[i]) for i in picks}
    with OraclePool(2) as pool:
        for key, c in cases.items():
            pool.submit(key, c, params, want_blob=(key == "t9"))
        # a 16-bit case: weights travel as float16
        c16 = (cases["t5"][0].astype(np.float16), cases["t5"][1].astype(np.float16), cases["t5"][2], cases["t5"][3])
        pool.submit("h5", c16, dict(params, flags=O.FLAG_W_F16))
        for key, c in list(cases.items()) + [("h5", c16)]:
            r = pool.result(key)
            ref = O.compress_step(*c, params["alpha"], params["beta"], 4, 3, flags=O.FLAG_W_F16 if key == "h5" else 0)
            assert (r["n"], r["n_w"], r["n_o"], r["nbytes"]) == (ref.n, ref.n_w, ref.n_o, len(ref.blob))
            assert r["blob_sha"] == hashlib.sha256(ref.blob).hexdigest()
            assert r["W_sha"] == digest(ref.W_recon) and r["m_sha"] == digest(ref.m_recon) and r["v_sha"] == digest(ref.v_recon)
            assert r["median"] == np.float32(ref.median).tobytes() and r["abs_sum_m"] == ref.abs_sum_m
            assert r["books"]["w"] == ref.C["w"].tobytes()
            assert ("blob" in r) == (key == "t9")
        assert pool.outstanding() == 0
