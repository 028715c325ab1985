"""Plain CPU oracle of the ExCP per-tensor compress / reconstruct step.

TEST INFRASTRUCTURE ONLY -- never on the product path, shares no code with the
HIP library, and is deliberately slow and literal so that every line can be
checked against the paper by eye.

Naming.  The paper's symbols for the two Adam moments are swapped relative to
standard Adam (Sec. 3: the "first-order and second-order moments v_t, m_t").
Here, as in the C ABI, ``m`` is the FIRST moment (signed EMA of the gradient)
and ``v`` is the SECOND moment (EMA of the squared gradient, non-negative):

    paper m_t (under the square root of Eq. "r_w")  ->  v  here
    paper v_t (the indicator of Eq. "r_o")          ->  m  here

All "fp32" arithmetic below is IEEE-754 binary32, round-to-nearest-even, one
rounding per operation (numpy float32 scalars/arrays), denormals preserved.

Pins.  Every function below is pinned by tests that do not re-use its own
formula: full-sort / counting invariants for the median, rational arithmetic
for the mean, element-by-element pure-Python brute force for the masks,
exhaustive nearest-centre search and a monotone objective for Lloyd, the
Lloyd iterations of two libraries started from the same centres (scipy's
kmeans2, scikit-learn's KMeans), textbook Lloyd-Max levels, uniform-data fixed
points, byte-level hand-built blobs and the size identities of the paper's
result tables.  The paper does not specify k-means initialisation, iteration
count, tie handling or empty-cluster handling (Sec. 3.3 says only "K-means
algorithm"): the choices made in ``kmeans_init`` / ``lloyd`` are this build's
reading, so which codebook is the right one is "parity unpinned" by the paper
itself; under that reading the values are pinned as listed above.
"""
from __future__ import annotations

import math
import struct
from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "MAGIC", "VERSION", "HEADER_BYTES", "FLAG_MEDIAN_OF_WEIGHTS", "FLAG_NO_M2W", "FLAG_NO_QUANT", "FLAG_NO_W2M", "FLAG_W_F16", "FLAG_W_BF16", "widen", "narrow",
    "RAW_BITS",
    "residual", "lower_median_abs", "exact_mean_abs", "weight_mask",
    "momentum_mask", "kmeans_init", "nearest_centre", "lloyd", "objective",
    "pack_bitmap", "pack_codes", "unpack_bitmap", "unpack_codes",
    "blob_size", "build_blob", "parse_blob", "compress_step",
    "decompress_step", "reconstruct_chain", "dense_bytes", "head_bytes", "dense_pack", "dense_unpack",
    "export_dense", "decompress_dense", "CompressResult", "BlobError", "NonFiniteError",
]

FLAG_MEDIAN_OF_WEIGHTS = 1
FLAG_NO_M2W = 2
FLAG_NO_QUANT = 4           # Table "abl", "prune" without "quant": the survivors are stored as they are (fp32)
FLAG_NO_W2M = 8             # Table "vit", no weights-to-momentum check: M_o does not depend on M_w
FLAG_W_F16 = 16             # the weights (previous, current, reconstructed) are IEEE binary16 (Sec. 4.3: PanGu)
FLAG_W_BF16 = 32            # ... or bfloat16, held as uint16 bit patterns
FLAGS_ALL = 63
RAW_BITS = 32               # the "code" width written into the header of a blob without quantisation
MAGIC = 0x50435845          # bytes "EXCP" read as a little-endian u32
VERSION = 1
HEADER_BYTES = 80

f32 = np.float32


class BlobError(ValueError):
    """The byte string is not a well-formed compressed tensor."""


class NonFiniteError(ValueError):
    """An input array holds NaN or Inf."""


# --------------------------------------------------------------------------
# Weights stored in 16 bits.  The method itself is unchanged: every weight is widened to fp32
# (exact), all arithmetic is the fp32 arithmetic described above, and a reconstructed weight is the
# fp32 sum rounded once more, to nearest even, into the storage format.  Pruned positions keep the
# previous weight's bits.
# --------------------------------------------------------------------------
def _check_flags(flags: int) -> None:
    if not 0 <= flags <= FLAGS_ALL or (flags & FLAG_W_F16 and flags & FLAG_W_BF16):
        raise ValueError("unknown or contradictory flags")


def widen(a, flags: int) -> np.ndarray:
    if flags & FLAG_W_F16:
        a = np.ascontiguousarray(a).ravel()
        assert a.dtype == np.float16
        return a.astype(f32)
    if flags & FLAG_W_BF16:
        a = np.ascontiguousarray(a).ravel()
        assert a.dtype == np.uint16
        return (a.astype(np.uint32) << np.uint32(16)).view(f32)
    return np.ascontiguousarray(a, dtype=f32).ravel()


def narrow(x: np.ndarray, flags: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=f32)
    if flags & FLAG_W_F16:
        with np.errstate(over="ignore"):
            return x.astype(np.float16)                       # IEEE round to nearest even
    if flags & FLAG_W_BF16:
        b = x.view(np.uint32).astype(np.uint64)
        assert not np.any(np.isnan(x))
        # drop 16 bits, nearest even: add half of the dropped range minus one, plus the kept lsb
        return ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)
    return x


# --------------------------------------------------------------------------
# Sec. 3.1, Eq. "ckpt_res"; Alg. 1 step 1
# --------------------------------------------------------------------------
def residual(W_prev: np.ndarray, W: np.ndarray) -> np.ndarray:
    """d = W_t - W_hat_{t-1}, one fp32 subtraction per element."""
    return (W.astype(f32, copy=False) - W_prev.astype(f32, copy=False)).astype(f32)


# --------------------------------------------------------------------------
# Sec. 3.2, Eq. "r_w": median(W), read as the median of |residual| of this
# tensor; an even-length tensor takes the LOWER middle element so that the
# result is one exact order statistic.
# --------------------------------------------------------------------------
def lower_median_abs(d: np.ndarray) -> np.float32:
    a = np.sort(np.abs(d.astype(f32, copy=False)), kind="stable")
    return f32(a[(a.size - 1) // 2])


# --------------------------------------------------------------------------
# Sec. 3.2, Eq. "r_o": mean(v_t), read as mean(|first moment|) over all n
# elements.  The sum is the exact real-number sum, rounded once to fp64, so
# the value does not depend on the order of summation.
# --------------------------------------------------------------------------
def exact_mean_abs(m: np.ndarray) -> tuple[float, np.float32]:
    a = np.abs(m.astype(f32, copy=False)).astype(np.float64)   # exact widening
    S = math.fsum(a.tolist())               # correctly rounded exact sum
    mean64 = S / float(a.size)
    return S, f32(mean64)


# --------------------------------------------------------------------------
# Sec. 3.2, Eq. "r_w": r_w(i) = alpha / sqrt(second moment_i) * median ;
# M_w(i) = [ |d_i| > r_w(i) ]  ("prune the residual ... by magnitude").
# Evaluation order fixed as (alpha*med) / sqrt(v_i), three fp32 roundings.
# v_i == 0 -> r = +inf -> pruned.  v_i < 0 -> sqrt = NaN -> comparison false.
# --------------------------------------------------------------------------
def weight_mask(d: np.ndarray, v: np.ndarray, alpha, med, use_moment: bool = True) -> tuple[np.ndarray, np.float32]:
    """``use_moment=False`` is the ablation of Table "vit" without the momentum-to-weights check:
    the threshold is the scalar alpha * med for every element."""
    t_w = f32(f32(alpha) * f32(med))
    if not use_moment:
        return np.abs(d.astype(f32, copy=False)) > t_w, t_w
    with np.errstate(divide="ignore", invalid="ignore", over="ignore", under="ignore"):
        root = np.sqrt(v.astype(f32, copy=False)).astype(f32)
        r = (t_w / root).astype(f32)
        Mw = np.abs(d.astype(f32, copy=False)) > r
    return Mw, t_w


# --------------------------------------------------------------------------
# Sec. 3.2, Eq. "r_o": r_o = beta * mean ; M_o(i) = [ |m_i| > r_o and M_w(i) ].
# --------------------------------------------------------------------------
def momentum_mask(m: np.ndarray, Mw: np.ndarray, beta, mean32) -> tuple[np.ndarray, np.float32]:
    r_o = f32(f32(beta) * f32(mean32))
    Mo = Mw & (np.abs(m.astype(f32, copy=False)) > r_o)
    return Mo, r_o


# --------------------------------------------------------------------------
# Sec. 3.3: k-means of the surviving values into 2^n - 1 centres.
# Initialisation (paper silent): the K order statistics at ranks
# ((2k+1) * len(x)) // (2K), k = 0..K-1 -- deterministic, sorted, no RNG.
# --------------------------------------------------------------------------
def kmeans_init(x: np.ndarray, K: int) -> np.ndarray:
    n = int(x.size)
    if n == 0:
        return np.zeros(K, dtype=f32)
    xs = np.sort(x.astype(f32, copy=False), kind="stable")
    idx = [((2 * k + 1) * n) // (2 * K) for k in range(K)]
    return xs[idx].astype(f32)


def nearest_centre(x: np.ndarray, C: np.ndarray) -> np.ndarray:
    """Index of the nearest centre of each x_j, for centres in ascending order.

    In one dimension the nearest centre is one of the two that bracket x_j.  With a = the last
    centre <= x_j and b = the next one (a = b at either end), the distances x_j - C_a and
    C_b - x_j are each evaluated in fp64 (one rounding); b wins only if it is strictly nearer,
    and among centres of equal value the lowest index is taken.  Evaluating all K distances in
    fp64 instead would not be equivalent: for a value far above every centre the rounded
    distances all coincide and the tie would send it to centre 0."""
    C64 = C.astype(np.float64)
    K = C64.size
    assert np.all(np.diff(C64) >= 0), "centres must be non-decreasing"
    x64 = x.astype(np.float64)
    j = np.searchsorted(C64, x64, side="right") - 1          # last centre <= x, or -1
    a = np.maximum(j, 0)
    b = np.minimum(j + 1, K - 1)
    da = np.abs(x64 - C64[a])
    db = np.abs(C64[b] - x64)
    pick = np.where(db < da, b, a)
    return np.searchsorted(C64, C64[pick], side="left").astype(np.int64)   # lowest index of that value


def objective(x: np.ndarray, C: np.ndarray, a: np.ndarray) -> float:
    """Sum over j of (x_j - C[a_j])^2, each term in fp64, exact summation."""
    if x.size == 0:
        return 0.0
    diff = x.astype(np.float64) - C.astype(np.float64)[a]
    return math.fsum((diff * diff).tolist())


def lloyd(x: np.ndarray, K: int, iters: int, history: list | None = None):
    """Exactly ``iters`` Lloyd updates from the quantile initialisation.

    update: C_k = fp32( exact sum of the members (rounded once to fp64) / count )
    for every non-empty cluster; an empty cluster keeps its centre.  Clusters are
    intervals of the sorted values, so the centres normally stay in ascending order;
    the one exception is a run of EQUAL centres (heavily tied data): the lowest of them
    takes all their members and may move past the ones that stay behind.  The centres
    are therefore put back in ascending order after every update (a stable sort, a
    no-op in the normal case); a codebook is a set of values, the order carries nothing.
    Returns (C fp32[K], a int64[len(x)]) where a is the assignment to the FINAL
    centres.  If ``history`` is a list, the objective before each update and
    after the last one is appended to it.
    """
    x = x.astype(f32, copy=False)
    C = kmeans_init(x, K)
    if x.size == 0:
        return C, np.empty(0, dtype=np.int64)
    x64 = x.astype(np.float64)
    for _ in range(iters):
        a = nearest_centre(x, C)
        if history is not None:
            history.append(objective(x, C, a))
        newC = C.copy()
        order = np.argsort(a, kind="stable")
        counts = np.bincount(a, minlength=K)
        pos = 0
        xsorted = x64[order]
        for k in range(K):
            c = int(counts[k])
            if c:
                S = math.fsum(xsorted[pos:pos + c].tolist())
                newC[k] = f32(S / float(c))
            pos += c
        C = np.sort(newC, kind="stable")
    a = nearest_centre(x, C)
    if history is not None:
        history.append(objective(x, C, a))
    return C, a


# --------------------------------------------------------------------------
# Packed representations (Sec. 4.2: "combine two int4 number into one int8").
# Bit i&63 of word i>>6 holds mask[i]; code j occupies bits
# [j*nbits, (j+1)*nbits) of the little-endian bit stream (earlier element in
# the lower bits), stored as little-endian u64 words.
# --------------------------------------------------------------------------
def _bits_to_words(bits: np.ndarray) -> np.ndarray:
    """Little-endian bit stream (bit j of the stream = bits[j]) -> u64 words."""
    nwords = (bits.size + 63) // 64
    padded = np.zeros(nwords * 64, dtype=np.uint8)
    padded[:bits.size] = bits
    return np.packbits(padded, bitorder="little").view("<u8").astype(np.uint64)


def _words_to_bits(words: np.ndarray, nbits_total: int) -> np.ndarray:
    raw = np.ascontiguousarray(words.astype("<u8")).view(np.uint8)
    return np.unpackbits(raw, bitorder="little")[:nbits_total]


def pack_bitmap(mask: np.ndarray) -> np.ndarray:
    return _bits_to_words(mask.astype(np.uint8))


def unpack_bitmap(words: np.ndarray, n: int) -> np.ndarray:
    return _words_to_bits(words, n).astype(bool)


def pack_codes(codes: np.ndarray, nbits: int) -> np.ndarray:
    codes = codes.astype(np.int64)
    assert codes.size == 0 or (codes.min() >= 0 and codes.max() < (1 << nbits))
    bits = ((codes[:, None] >> np.arange(nbits)[None, :]) & 1).astype(np.uint8)
    return _bits_to_words(bits.reshape(-1))


def unpack_codes(words: np.ndarray, n: int, nbits: int) -> np.ndarray:
    bits = _words_to_bits(words, n * nbits).reshape(n, nbits).astype(np.int64)
    return (bits << np.arange(nbits)[None, :]).sum(axis=1)


def _pad16(nbytes: int) -> int:
    return (nbytes + 15) // 16 * 16


def blob_size(n: int, n_w: int, n_o: int, nbits: int, flags: int = 0) -> int:
    """Closed-form size of one compressed tensor (bytes).  nbits = RAW_BITS: no codebooks, fp32 values
    in place of codes; FLAG_NO_W2M: the second bitmap covers all n elements, not the n_w survivors."""
    size = HEADER_BYTES + (0 if nbits == RAW_BITS else 3 * 4 * (1 << nbits))
    size += _pad16(8 * ((n + 63) // 64))
    size += _pad16(8 * (((n if flags & FLAG_NO_W2M else n_w) + 63) // 64))
    size += _pad16(8 * ((n_w * nbits + 63) // 64))
    size += 2 * _pad16(8 * ((n_o * nbits + 63) // 64))
    return size


def _section(words: np.ndarray) -> bytes:
    raw = words.astype("<u8").tobytes()
    return raw + b"\0" * (_pad16(len(raw)) - len(raw))


def build_blob(*, n, nbits, flags, iters, alpha, beta, med, mean32, t_w, r_o,
               Cw, Cm, Cv, Mw, Mo_over_survivors, codes_w, codes_m, codes_v) -> bytes:
    n_w = int(Mw.sum())
    n_o = int(Mo_over_survivors.sum())
    assert Mo_over_survivors.size == (n if flags & FLAG_NO_W2M else n_w)
    total = blob_size(n, n_w, n_o, nbits, flags)
    head = struct.pack("<IIIIQQQffffffQII",
                       MAGIC, VERSION, nbits, flags, n, n_w, n_o,
                       float(f32(alpha)), float(f32(beta)), float(med), float(mean32),
                       float(t_w), float(r_o), total, iters, 0)
    assert len(head) == HEADER_BYTES
    parts = [head]
    for C in (Cw, Cm, Cv):
        if nbits == RAW_BITS:
            break                                            # nothing is quantised: no codebooks
        book = np.concatenate([np.zeros(1, dtype=f32), C.astype(f32)])
        parts.append(book.astype("<f4").tobytes())
    parts.append(_section(pack_bitmap(Mw)))
    parts.append(_section(pack_bitmap(Mo_over_survivors)))
    parts.append(_section(pack_codes(codes_w, nbits)))
    parts.append(_section(pack_codes(codes_m, nbits)))
    parts.append(_section(pack_codes(codes_v, nbits)))
    blob = b"".join(parts)
    assert len(blob) == total
    return blob


def parse_blob(blob: bytes, n_expected: int | None = None) -> dict:
    if len(blob) < HEADER_BYTES:
        raise BlobError("shorter than a header")
    (magic, version, nbits, flags, n, n_w, n_o, alpha, beta, med, mean32, t_w, r_o,
     total, iters, reserved) = struct.unpack("<IIIIQQQffffffQII", blob[:HEADER_BYTES])
    if magic != MAGIC:
        raise BlobError("bad magic")
    if version != VERSION:
        raise BlobError("bad version")
    if flags > FLAGS_ALL or (flags & FLAG_W_F16 and flags & FLAG_W_BF16):
        raise BlobError("unknown flags")
    if not (2 <= nbits <= 8 or (nbits == RAW_BITS and flags & FLAG_NO_QUANT)) or \
            (nbits != RAW_BITS and flags & FLAG_NO_QUANT):
        raise BlobError("nbits out of range")
    if n_expected is not None and n != n_expected:
        raise BlobError("element count mismatch")
    if not (n_w <= n and n_o <= (n if flags & FLAG_NO_W2M else n_w)):
        raise BlobError("inconsistent counts")
    if total != blob_size(n, n_w, n_o, nbits, flags) or len(blob) < total:
        raise BlobError("inconsistent size")
    E = 0 if nbits == RAW_BITS else 1 << nbits
    off = HEADER_BYTES
    books = []
    for _ in range(3):
        books.append(np.frombuffer(blob, dtype="<f4", count=E, offset=off).astype(f32))
        off += 4 * E

    def take(nwords):
        nonlocal off
        arr = np.frombuffer(blob, dtype="<u8", count=nwords, offset=off).astype(np.uint64)
        off += _pad16(8 * nwords)
        return arr

    bw = take((n + 63) // 64)
    bo = take(((n if flags & FLAG_NO_W2M else n_w) + 63) // 64)
    cw = take((n_w * nbits + 63) // 64)
    cm = take((n_o * nbits + 63) // 64)
    cv = take((n_o * nbits + 63) // 64)
    return dict(nbits=nbits, flags=flags, n=n, n_w=n_w, n_o=n_o, alpha=f32(alpha),
                beta=f32(beta), median=f32(med), mean_abs_m=f32(mean32), t_w=f32(t_w),
                r_o=f32(r_o), blob_bytes=total, iters=iters,
                book_w=books[0], book_m=books[1], book_v=books[2],
                bitmap_w=bw, bitmap_o=bo, codes_w=cw, codes_m=cm, codes_v=cv)


@dataclass
class CompressResult:
    blob: bytes
    W_recon: np.ndarray
    m_recon: np.ndarray
    v_recon: np.ndarray
    n: int
    n_w: int
    n_o: int
    median: np.float32
    abs_sum_m: float
    mean_abs_m: np.float32
    t_w: np.float32
    r_o: np.float32
    Mw: np.ndarray
    Mo: np.ndarray
    C: dict = field(default_factory=dict)        # stream -> fp32[K] centres
    assign: dict = field(default_factory=dict)   # stream -> int64 assignment (0-based)
    obj: dict = field(default_factory=dict)      # stream -> final objective
    x: dict = field(default_factory=dict)        # stream -> surviving values

    @property
    def ratio(self) -> float:
        return 12.0 * self.n / len(self.blob)


# --------------------------------------------------------------------------
# Alg. 1 (without the final general-purpose archive stage) for one tensor.
# --------------------------------------------------------------------------
def compress_step(W_prev, W, m, v, alpha=5e-5, beta=2.0, nbits=4, iters=10,
                  flags=0) -> CompressResult:
    _check_flags(flags)
    W_prev_stored = np.ascontiguousarray(W_prev).ravel()
    W_prev = widen(W_prev, flags)
    W = widen(W, flags)
    m = np.ascontiguousarray(m, dtype=f32).ravel()
    v = np.ascontiguousarray(v, dtype=f32).ravel()
    n = W.size
    assert W_prev.size == n and m.size == n and v.size == n
    assert 2 <= nbits <= 8 and iters >= 0
    raw = bool(flags & FLAG_NO_QUANT)
    stored_bits = RAW_BITS if raw else nbits
    for arr in (W_prev, W, m, v):
        if not np.all(np.isfinite(arr)):
            raise NonFiniteError("NaN or Inf in an input")
    K = (1 << nbits) - 1

    if n == 0:
        z = np.zeros(0, dtype=f32)
        zb = np.zeros(0, dtype=bool)
        zc = np.zeros(0, dtype=np.int64)
        C0 = np.zeros(K, dtype=f32)
        blob = build_blob(n=0, nbits=stored_bits, flags=flags, iters=iters, alpha=alpha, beta=beta,
                          med=f32(0), mean32=f32(0), t_w=f32(0), r_o=f32(0),
                          Cw=C0, Cm=C0, Cv=C0, Mw=zb, Mo_over_survivors=zb,
                          codes_w=zc, codes_m=zc, codes_v=zc)
        return CompressResult(blob, narrow(z, flags), z, z, 0, 0, 0, f32(0), 0.0, f32(0), f32(0), f32(0),
                              zb, zb, dict(w=C0, m=C0, v=C0), dict(w=zc, m=zc, v=zc),
                              dict(w=0.0, m=0.0, v=0.0), dict(w=z, m=z, v=z))

    with np.errstate(over="ignore"):
        d = residual(W_prev, W)                               # Alg. 1 step 1
    if not np.all(np.isfinite(d)):
        raise NonFiniteError("the residual overflows fp32")
    # flags: bit 0 = the median of Eq. r_w is taken over |W_t| instead of the residual (the other
    # reading of "median(W)"); bit 1 = no momentum-to-weights check (Table "vit"): scalar threshold
    med = lower_median_abs(W if flags & FLAG_MEDIAN_OF_WEIGHTS else d)      # Eq. r_w
    S, mean32 = exact_mean_abs(m)                             # Eq. r_o
    Mw, t_w = weight_mask(d, v, alpha, med, use_moment=not (flags & FLAG_NO_M2W))   # Eq. r_w
    # bit 3: without the weights-to-momentum check the moment mask of Eq. r_o stands on its own
    w2m = not (flags & FLAG_NO_W2M)
    Mo, r_o = momentum_mask(m, Mw if w2m else np.ones(n, dtype=bool), beta, mean32)   # Eq. r_o
    xw, xm, xv = d[Mw], m[Mo], v[Mo]                          # survivors, index order

    C, A, O = {}, {}, {}
    stored = {}
    for name, x in (("w", xw), ("m", xm), ("v", xv)):         # Alg. 1 steps 3-4
        if raw:                                               # bit 2: no quantisation, the values themselves
            C[name], A[name], O[name] = np.zeros(0, dtype=f32), None, 0.0
            stored[name] = x.copy()
            codes = x.view(np.uint32).astype(np.int64)
        else:
            C[name], A[name] = lloyd(x, K, iters)
            O[name] = objective(x, C[name], A[name])
            stored[name] = C[name][A[name]]
            codes = A[name] + 1
        stored[name + "_codes"] = codes

    blob = build_blob(n=n, nbits=stored_bits, flags=flags, iters=iters, alpha=alpha, beta=beta,
                      med=med, mean32=mean32, t_w=t_w, r_o=r_o,
                      Cw=C["w"], Cm=C["m"], Cv=C["v"], Mw=Mw, Mo_over_survivors=Mo[Mw] if w2m else Mo,
                      codes_w=stored["w_codes"], codes_m=stored["m_codes"], codes_v=stored["v_codes"])

    # Alg. 2 applied to what was just stored (the copy kept for the next step).
    W_rec = _apply_residual(W_prev_stored, W_prev, np.flatnonzero(Mw), stored["w"], flags)
    m_rec = np.zeros(n, dtype=f32)
    v_rec = np.zeros(n, dtype=f32)
    m_rec[Mo] = stored["m"]
    v_rec[Mo] = stored["v"]
    return CompressResult(blob, W_rec, m_rec, v_rec, n, int(Mw.sum()), int(Mo.sum()),
                          med, S, mean32, t_w, r_o, Mw, Mo, C, A, O,
                          dict(w=xw, m=xm, v=xv))


def _apply_residual(W_prev_stored, W_prev32, idx, values, flags):
    """W_hat: the previous weights with `values` added at `idx` (fp32 addition, then the storage
    format's rounding when the weights are 16-bit); everything else keeps its bits."""
    out = np.array(W_prev_stored, copy=True)
    out[idx] = narrow((W_prev32[idx] + values).astype(f32), flags)
    return out


# --------------------------------------------------------------------------
# Alg. 2 for one tensor, from the stored bytes alone.
# --------------------------------------------------------------------------
def decompress_step(W_prev, blob: bytes):
    flags = parse_blob(blob)["flags"]
    W_prev_stored = np.ascontiguousarray(W_prev).ravel()
    W_prev = widen(W_prev, flags)
    p = parse_blob(blob, n_expected=W_prev.size)
    n, n_w, n_o, nbits = p["n"], p["n_w"], p["n_o"], p["nbits"]
    idx_w, idx_o = _kept_indices(p)
    vals = []
    for key, count in (("w", n_w), ("m", n_o), ("v", n_o)):
        c = unpack_codes(p["codes_" + key], count, nbits)
        if nbits == RAW_BITS:
            vals.append(c.astype(np.uint32).view(f32))              # stored as they were
        else:
            vals.append(p["book_" + key][c])                        # Alg. 2 steps 2-3: codebook look-up
    W_rec = _apply_residual(W_prev_stored, W_prev, idx_w, vals[0], flags)   # Alg. 2 step 4
    m_rec = np.zeros(n, dtype=f32)
    v_rec = np.zeros(n, dtype=f32)
    m_rec[idx_o] = vals[1]
    v_rec[idx_o] = vals[2]
    return W_rec, m_rec, v_rec


def _kept_indices(p: dict):
    """Element indices of the kept residuals and of the kept moment pairs of a parsed blob."""
    n, n_w, n_o = p["n"], p["n_w"], p["n_o"]
    Mw = unpack_bitmap(p["bitmap_w"], n)
    idx_w = np.flatnonzero(Mw)
    if p["flags"] & FLAG_NO_W2M:
        Mo = unpack_bitmap(p["bitmap_o"], n)                        # over all elements
        idx_o = np.flatnonzero(Mo)
    else:
        Mo = unpack_bitmap(p["bitmap_o"], n_w)                      # over the kept residuals
        idx_o = idx_w[Mo[:idx_w.size]] if idx_w.size == n_w else idx_w[:0]
    if idx_w.size != n_w or int(Mo.sum()) != n_o:
        raise BlobError("bitmap population does not match the header")
    return idx_w, idx_o


def reconstruct_chain(W0, blobs):
    """Alg. 3: from the weights the chain starts with, apply the compressed checkpoints one after the
    other (each is Alg. 2 against the reconstruction before it).  Returns the last reconstruction and
    the moments stored in the last checkpoint."""
    W = np.ascontiguousarray(W0).ravel()
    m = v = None
    for blob in blobs:
        W, m, v = decompress_step(W, blob)
    return W, m, v


# --------------------------------------------------------------------------
# The stored layout of Sec. 4.2: one code per ELEMENT (0 = pruned, 1..K = centre index + 1), the
# codes of 4 bits or fewer two to a byte, handed to a general-purpose archiver (Alg. 1, last step).
# The paper does not say which element takes which half of the byte: here the even element takes
# the low four bits.  Codes wider than four bits take one byte each.
# --------------------------------------------------------------------------
def dense_bytes(n: int, nbits: int) -> int:
    return (n + 1) // 2 if nbits <= 4 else n


def head_bytes(nbits: int) -> int:
    """Header and the three codebooks: the leading bytes of a blob, kept verbatim beside the codes."""
    return HEADER_BYTES + 12 * (1 << nbits)


def dense_pack(codes: np.ndarray, nbits: int) -> np.ndarray:
    codes = np.asarray(codes, dtype=np.int64)
    assert codes.size == 0 or (codes.min() >= 0 and codes.max() < (1 << nbits))
    if nbits > 4:
        return codes.astype(np.uint8)
    padded = np.zeros(2 * dense_bytes(codes.size, nbits), dtype=np.int64)     # an odd tail pairs with code 0
    padded[:codes.size] = codes
    return (padded[0::2] + 16 * padded[1::2]).astype(np.uint8)


def dense_unpack(packed: np.ndarray, n: int, nbits: int) -> np.ndarray:
    packed = np.asarray(packed, dtype=np.uint8)
    if packed.size != dense_bytes(n, nbits):
        raise BlobError("wrong length of a code tensor")
    if nbits > 4:
        return packed.astype(np.int64)
    both = np.empty(2 * packed.size, dtype=np.int64)
    both[0::2] = packed & 15
    both[1::2] = packed >> 4
    if n % 2 == 1 and both[n] != 0:
        raise BlobError("the unused half of the last byte is not zero")
    return both[:n]


def export_dense(blob: bytes):
    """Blob -> (head, codes_w, codes_m, codes_v): the per-element code tensors of Sec. 4.2."""
    p = parse_blob(blob)
    n, n_w, n_o, nbits = p["n"], p["n_w"], p["n_o"], p["nbits"]
    if nbits == RAW_BITS:
        raise BlobError("a blob without quantisation has no codes to export")
    idx_w, idx_o = _kept_indices(p)
    per_element = []
    for idx, words, count in ((idx_w, p["codes_w"], n_w), (idx_o, p["codes_m"], n_o), (idx_o, p["codes_v"], n_o)):
        e = np.zeros(n, dtype=np.int64)                      # pruned elements keep code 0
        e[idx] = unpack_codes(words, count, nbits)
        per_element.append(dense_pack(e, nbits))
    return bytes(blob[:head_bytes(nbits)]), per_element[0], per_element[1], per_element[2]


def decompress_dense(W_prev, head: bytes, codes_w, codes_m, codes_v):
    """Alg. 2 from the stored layout of Sec. 4.2: look every element's code up in its codebook; code 0
    leaves the previous weight untouched and gives a zero moment."""
    if len(head) < HEADER_BYTES:
        raise BlobError("shorter than a header")
    magic, version, nbits, flags, n_stored = struct.unpack("<IIIIQ", head[:24])
    if flags > FLAGS_ALL or (flags & FLAG_W_F16 and flags & FLAG_W_BF16):
        raise BlobError("bad header")
    W_prev_stored = np.ascontiguousarray(W_prev).ravel()
    W_prev = widen(W_prev, flags)
    n = W_prev.size
    if magic != MAGIC or version != VERSION or not 2 <= nbits <= 8 or n_stored != n:
        raise BlobError("bad header")
    if len(head) < head_bytes(nbits):
        raise BlobError("codebooks missing")
    E = 1 << nbits
    books = [np.frombuffer(head, dtype="<f4", count=E, offset=HEADER_BYTES + 4 * E * k).astype(f32) for k in range(3)]
    out = []
    for k, packed in enumerate((codes_w, codes_m, codes_v)):
        c = dense_unpack(packed, n, nbits)
        if c.size and c.max() > E - 1:
            raise BlobError("code beyond the codebook")
        kept = c != 0
        if k == 0:
            r = _apply_residual(W_prev_stored, W_prev, np.flatnonzero(kept), books[0][c[kept]], flags)
        else:
            r = np.zeros(n, dtype=f32)
            r[kept] = books[k][c[kept]]
        out.append(r)
    return out[0], out[1], out[2]

