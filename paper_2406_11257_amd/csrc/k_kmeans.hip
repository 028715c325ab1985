// Non-uniform quantisation of the surviving values (Sec. 3.3): per stream, K = 2^nbits - 1
// centres by Lloyd's algorithm, then codes = 1 + nearest centre packed nbits each (Sec. 4.2).
//
// One-dimensional Lloyd has structure that makes re-reading every value in every iteration
// unnecessary: clusters are intervals, and the assignment is monotone in the value.  So each stream
// is first PARTITIONED into 256 value-ordered buckets of roughly equal population (splitters from a
// sorted sample), and for every bucket the exact count, exact sum, minimum and maximum are stored.
// In an iteration a bucket whose minimum and maximum go to the same centre contributes its stored
// totals; only the (at most K-1) buckets that a cluster border cuts are read element by element.
// The same buckets give the initial centres (order statistics of rank ((2k+1) len)/(2K)) with a
// radix select inside one bucket per rank.
//
// All sums are exact: a value is mant * 2^(pos-149); mantissas are added as integers in windows of
// 40 binary orders and filed into signed 64-bit bins 8 binary orders apart (the representation of
// the exact sum of |m| in the statistics pass, here with sign).  A centre is therefore
// fp32(round-once-fp64(exact sum) / count), independent of the order in which values were met, so
// integer atomics may be used freely and the partition need not be stable.
//
// The survivor passes walk one chunk list (8192 values per chunk) spanning every stream of every
// tensor of the group; its length is known only on the device.
#include "excp_util.h"

namespace {

constexpr u32 NBKT = 256;
constexpr u32 SAMPLE = 4096;
constexpr u32 PER_THREAD = EXCP_CHUNK / EXCP_THREADS;   // 32

__device__ __forceinline__ const float *seg_data(const Workspace &w, u32 sidx) {
    const u32 t = sidx / 3u, which = sidx % 3u;
    const float *basep = which == 0 ? w.xw : (which == 1 ? w.xm : w.xv);
    return basep + w.desc[t].elem_off;
}
__device__ __forceinline__ float *seg_part(const Workspace &w, u32 sidx) {
    const u32 t = sidx / 3u, which = sidx % 3u;
    float *basep = which == 0 ? w.pw : (which == 1 ? w.pm : w.pv);
    return basep + w.desc[t].elem_off;
}

// number of splitters (split[0..254]) that are <= key: the bucket of key, 0..255
__device__ __forceinline__ u32 bucket_of(const u32 *split, u32 key) {
    u32 lo = 0;
#pragma unroll
    for (u32 step = 128; step >= 1; step >>= 1) {
        u32 probe = lo + step - 1;                 // <= 254
        if (split[probe] <= key) lo += step;
    }
    return lo < 255u ? lo : 255u;
}

// The same search for N keys at once, step by step: the N LDS reads of a step are independent and
// overlap, instead of N chains of eight dependent reads.
template <int N>
__device__ __forceinline__ void bucket_of_many(const u32 *split, const u32 (&key)[N], u32 (&out)[N]) {
#pragma unroll
    for (int e = 0; e < N; ++e) out[e] = 0;
#pragma unroll
    for (u32 step = 128; step >= 1; step >>= 1) {
        u32 probe[N];
#pragma unroll
        for (int e = 0; e < N; ++e) probe[e] = split[out[e] + step - 1];
#pragma unroll
        for (int e = 0; e < N; ++e) if (probe[e] <= key[e]) out[e] += step;
    }
#pragma unroll
    for (int e = 0; e < N; ++e) out[e] = out[e] < 255u ? out[e] : 255u;
}

// ---------------------------------------------------------------- exact signed accumulation
// Adds the values x[j] (j < N) with sel[j] set, for the whole wave, to a set of signed bins through
// add(bin, delta): sum_g bins[g] * 2^(8g-149) grows by exactly the sum of the selected values.
template <int N, class Add>
__device__ __forceinline__ void wave_exact_add(const float (&x)[N], const bool (&sel)[N], Add add) {
    const u32 lane = lane_id();
    u32 pmax = 0, any = 0;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        u32 mb = f2u(x[j]) & 0x7fffffffu;
        u32 e = mb >> 23;
        u32 pos = (e ? e : 1u) - 1u;
        if (sel[j] && mb) { pmax = max(pmax, pos); any = 1; }
    }
    if (!__any(any)) return;
    pmax = wave_max_u32(pmax);
    const u32 B = pmax > 39u ? pmax - 39u : 0u;
    u64 pL = 0, pH = 0, nL = 0, nH = 0;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        u32 u = f2u(x[j]);
        u32 mb = u & 0x7fffffffu;
        u32 e = mb >> 23;
        u32 mant = (mb & 0x7fffffu) | (e ? 0x800000u : 0u);
        u32 pos = (e ? e : 1u) - 1u;
        if (sel[j] && mant) {
            const bool neg = u >> 31;
            if (pos >= B) {
                u64 term = (u64)mant << (pos - B);
                if (neg) { nL += term & 0xffffffffull; nH += term >> 32; }
                else { pL += term & 0xffffffffull; pH += term >> 32; }
            } else {
                u64 d = (u64)mant << (pos & 7u);
                add(pos >> 3, neg ? (u64)0 - d : d);
            }
        }
    }
#pragma unroll
    for (int sgn = 0; sgn < 2; ++sgn) {
        u64 aL = sgn ? nL : pL, aH = sgn ? nH : pH;
        if (!__any(aL != 0 || aH != 0)) continue;
        aL = wave_sum_u64(aL);
        aH = wave_sum_u64(aH);
        if (lane == 0) {
            u64 lo64 = aL + (aH << 32);
            u64 hi64 = (aH >> 32) + (lo64 < aL ? 1ull : 0ull);
            u64 piece[3] = {lo64 & 0xffffffffull, lo64 >> 32, hi64};
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                u32 p = B + 32u * q;
                if (piece[q]) { u64 d = piece[q] << (p & 7u); add(p >> 3, sgn ? (u64)0 - d : d); }
            }
        }
    }
}

// Signed bins -> the exact sum rounded once (to nearest, ties to even) to fp64.
__device__ double signed_bins_to_double(const u64 *bins) {
    u32 limb[14];
    for (int i = 0; i < 14; ++i) limb[i] = 0;
    for (int g = 0; g < EXCP_ABSM_BINS; ++g) {
        long long c = (long long)bins[g];
        if (!c) continue;
        // sign-extended 64-bit value shifted left by 8g, added into a 448-bit two's complement number
        u32 bit = 8u * g, li = bit >> 5, sh = bit & 31u;
        u32 ext = c < 0 ? 0xffffffffu : 0u;
        u64 uc = (u64)c;
        u64 carry = 0;
        for (u32 q = 0; li + q < 14; ++q) {
            // 32-bit slice q of (sign-extended c) << sh
            u32 lo_part, hi_part;
            auto word = [&](int idx) -> u32 { return idx < 0 ? 0u : (idx == 0 ? (u32)uc : (idx == 1 ? (u32)(uc >> 32) : ext)); };
            lo_part = word((int)q);
            hi_part = word((int)q - 1);
            u32 slice = sh ? ((lo_part << sh) | (hi_part >> (32 - sh))) : lo_part;
            u64 s = (u64)limb[li + q] + slice + carry;
            limb[li + q] = (u32)s;
            carry = s >> 32;
        }
    }
    const bool neg = limb[13] >> 31;
    if (neg) {                                  // magnitude = two's complement negation
        u64 carry = 1;
        for (int i = 0; i < 14; ++i) { u64 s = (u64)(~limb[i]) + carry; limb[i] = (u32)s; carry = s >> 32; }
    }
    int top = -1;
    for (int i = 13; i >= 0; --i) if (limb[i]) { top = i; break; }
    if (top < 0) return 0.0;
    int msb = 32 * top + (31 - __clz((int)limb[top]));
    auto bit_at = [&](int p) -> u32 { return p < 0 ? 0u : (limb[p >> 5] >> (p & 31)) & 1u; };
    double mag;
    if (msb <= 52) {
        u64 x = (u64)limb[0] | ((u64)limb[1] << 32);
        mag = ldexp((double)x, -149);
    } else {
        u64 mant = 0;
        for (int p = msb; p >= msb - 52; --p) mant = (mant << 1) | bit_at(p);
        u32 guard = bit_at(msb - 53), sticky = 0;
        for (int p = msb - 54; p >= 0 && !sticky; --p) sticky |= bit_at(p);
        if (guard && (sticky || (mant & 1ull))) mant += 1;
        mag = ldexp((double)mant, msb - 52 - 149);
    }
    return neg ? -mag : mag;
}

// ---------------------------------------------------------------- P0: splitters from a sorted sample
__global__ __launch_bounds__(EXCP_THREADS) void k_km_sample(Workspace w, GroupParams g) {
    __shared__ u32 key[SAMPLE];
    const u32 sidx = blockIdx.x, tid = threadIdx.x;
    const u64 len = w.seg[sidx].len;
    if (len == 0) return;
    const float *__restrict__ x = seg_data(w, sidx);
    const u32 ns = len < SAMPLE ? (u32)len : SAMPLE;
    for (u32 i = tid; i < SAMPLE; i += EXCP_THREADS)
        key[i] = (i < ns) ? key_of(x[((u64)i * len) / ns]) : 0xffffffffu;
    __syncthreads();
    for (u32 k = 2; k <= SAMPLE; k <<= 1) {
        for (u32 j = k >> 1; j > 0; j >>= 1) {
            for (u32 t = tid; t < SAMPLE / 2; t += EXCP_THREADS) {
                u32 i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                u32 p = i | j;
                u32 a = key[i], b = key[p];
                bool asc = (i & k) == 0;
                if ((a > b) == asc) { key[i] = b; key[p] = a; }
            }
            __syncthreads();
        }
    }
    u32 *split = w.km_split + (u64)sidx * NBKT;
    for (u32 b = tid; b < NBKT; b += EXCP_THREADS) {
        u32 idx = (u32)(((u64)(b + 1) * ns) / NBKT);
        if (idx >= ns) idx = ns - 1;
        split[b] = (b == NBKT - 1) ? 0xffffffffu : key[idx];
    }
}

// ---------------------------------------------------------------- P1: per-chunk bucket counts
__global__ __launch_bounds__(EXCP_THREADS) void k_km_count(Workspace w, GroupParams g) {
    __shared__ u32 split[NBKT];
    __shared__ u32 hist[NBKT];
    const u32 tid = threadIdx.x;
    const u32 total = *w.chunk_total;
    const u32 G = gridDim.x, b = blockIdx.x;
    const u32 lo = (u32)(((u64)b * total) / G), hi = (u32)(((u64)(b + 1) * total) / G);
    if (lo >= hi) return;
    const u32 nseg = 3u * g.ntensors;
    u32 sidx = 0xffffffffu, s_end = 0;
    for (u32 c = lo; c < hi; ++c) {
        if (sidx == 0xffffffffu || c >= s_end) {
            __syncthreads();
            sidx = find_owner(w.seg_chunk_begin, nseg, c);
            s_end = w.seg_chunk_begin[sidx + 1];
            split[tid] = w.km_split[(u64)sidx * NBKT + tid];
        }
        hist[tid] = 0;
        __syncthreads();
        const SegState &S = w.seg[sidx];
        const float *__restrict__ x = seg_data(w, sidx);
        const u64 len = S.len;
        const u64 base = (u64)(c - S.chunk_begin) * EXCP_CHUNK;
        const u32 clen = (len - base) < EXCP_CHUNK ? (u32)(len - base) : EXCP_CHUNK;
        const EXCP_GLOBAL float *gx = gptr(x) + base;
#pragma unroll
        for (u32 half = 0; half < 2; ++half) {
            u32 key[PER_THREAD / 2], bk[PER_THREAD / 2];
#pragma unroll
            for (u32 it = 0; it < PER_THREAD / 2; ++it) {
                const u32 e = (half * (PER_THREAD / 2) + it) * EXCP_THREADS + tid;
                key[it] = key_of(gx[e < clen ? e : 0]);
            }
            bucket_of_many<PER_THREAD / 2>(split, key, bk);
#pragma unroll
            for (u32 it = 0; it < PER_THREAD / 2; ++it) {
                const u32 e = (half * (PER_THREAD / 2) + it) * EXCP_THREADS + tid;
                if (e < clen) atomicAdd(&hist[bk[it]], 1u);
            }
        }
        __syncthreads();
        w.km_cnt[(u64)c * NBKT + tid] = hist[tid];
        __syncthreads();
    }
}

// ---------------------------------------------------------------- P2: offsets of every (chunk, bucket)
// 1024 threads: thread (q, b) owns bucket b over one quarter of the stream's chunks.
__global__ __launch_bounds__(1024) void k_km_scan(Workspace w, GroupParams g) {
    __shared__ u32 tot[4][NBKT];
    __shared__ u32 begin[NBKT + 1];
    const u32 sidx = blockIdx.x, tid = threadIdx.x, q = tid >> 8, b = tid & 255u;
    const u64 len = w.seg[sidx].len;
    if (len == 0) return;
    const u32 c0 = w.seg[sidx].chunk_begin, c1 = w.seg_chunk_begin[sidx + 1];
    const u32 nq = (c1 - c0 + 3) / 4;
    const u32 a0 = min(c0 + q * nq, c1), a1 = min(a0 + nq, c1);
    u32 *cnt = w.km_cnt;
    u32 s = 0;
#pragma unroll 8
    for (u32 c = a0; c < a1; ++c) s += cnt[(u64)c * NBKT + b];
    tot[q][b] = s;
    __syncthreads();
    if (q == 0) begin[b + 1] = tot[0][b] + tot[1][b] + tot[2][b] + tot[3][b];
    if (tid == 0) begin[0] = 0;
    __syncthreads();
    // inclusive scan of begin[1..256] by the first 256 threads
    for (u32 off = 1; off < NBKT; off <<= 1) {
        u32 v = 0;
        if (q == 0 && b >= off) v = begin[b + 1 - off];
        __syncthreads();
        if (q == 0) begin[b + 1] += v;
        __syncthreads();
    }
    if (q == 0) {
        w.km_begin[(u64)sidx * (NBKT + 1) + b + 1] = begin[b + 1];
        if (b == 0) w.km_begin[(u64)sidx * (NBKT + 1)] = 0;
    }
    u32 run = begin[b];
    for (u32 qq = 0; qq < q; ++qq) run += tot[qq][b];
#pragma unroll 4
    for (u32 c = a0; c < a1; ++c) {
        u32 v = cnt[(u64)c * NBKT + b];
        cnt[(u64)c * NBKT + b] = run;
        run += v;
    }
}

// ---------------------------------------------------------------- P3: scatter into buckets
__global__ __launch_bounds__(EXCP_THREADS) void k_km_scatter(Workspace w, GroupParams g) {
    __shared__ u32 split[NBKT];
    __shared__ u32 hist[NBKT], loff[NBKT], goff[NBKT], fill[NBKT];
    __shared__ float sval[EXCP_CHUNK];
    __shared__ unsigned char sbkt[EXCP_CHUNK];
    const u32 tid = threadIdx.x;
    const u32 total = *w.chunk_total;
    const u32 G = gridDim.x, bid = blockIdx.x;
    const u32 lo = (u32)(((u64)bid * total) / G), hi = (u32)(((u64)(bid + 1) * total) / G);
    if (lo >= hi) return;
    const u32 nseg = 3u * g.ntensors;
    u32 sidx = 0xffffffffu, s_end = 0;
    for (u32 c = lo; c < hi; ++c) {
        if (sidx == 0xffffffffu || c >= s_end) {
            __syncthreads();
            sidx = find_owner(w.seg_chunk_begin, nseg, c);
            s_end = w.seg_chunk_begin[sidx + 1];
            split[tid] = w.km_split[(u64)sidx * NBKT + tid];
        }
        hist[tid] = 0; fill[tid] = 0;
        goff[tid] = w.km_cnt[(u64)c * NBKT + tid];
        __syncthreads();
        const SegState &S = w.seg[sidx];
        const float *__restrict__ x = seg_data(w, sidx);
        float *__restrict__ part = seg_part(w, sidx);
        const u64 len = S.len;
        const u64 base = (u64)(c - S.chunk_begin) * EXCP_CHUNK;
        const u32 clen = (len - base) < EXCP_CHUNK ? (u32)(len - base) : EXCP_CHUNK;
        float v[PER_THREAD];
        u32 bk[PER_THREAD];
        const EXCP_GLOBAL float *gx = gptr(x) + base;
#pragma unroll
        for (u32 it = 0; it < PER_THREAD; ++it) {
            u32 e = it * EXCP_THREADS + tid;
            v[it] = gx[e < clen ? e : 0];
        }
#pragma unroll
        for (u32 half = 0; half < 2; ++half) {
            u32 key[PER_THREAD / 2], out[PER_THREAD / 2];
#pragma unroll
            for (u32 it = 0; it < PER_THREAD / 2; ++it) key[it] = key_of(v[half * (PER_THREAD / 2) + it]);
            bucket_of_many<PER_THREAD / 2>(split, key, out);
#pragma unroll
            for (u32 it = 0; it < PER_THREAD / 2; ++it) {
                const u32 e = (half * (PER_THREAD / 2) + it) * EXCP_THREADS + tid;
                bk[half * (PER_THREAD / 2) + it] = out[it];
                if (e < clen) atomicAdd(&hist[out[it]], 1u);
            }
        }
        __syncthreads();
        // exclusive scan of the 256 bucket counts
        {
            u32 mine = hist[tid];
            loff[tid] = mine;
            __syncthreads();
            for (u32 off = 1; off < NBKT; off <<= 1) {
                u32 a = (tid >= off) ? loff[tid - off] : 0u;
                __syncthreads();
                loff[tid] += a;
                __syncthreads();
            }
            u32 incl = loff[tid];
            __syncthreads();
            loff[tid] = incl - mine;
            __syncthreads();
        }
#pragma unroll
        for (u32 it = 0; it < PER_THREAD; ++it) {
            u32 e = it * EXCP_THREADS + tid;
            if (e < clen) {
                u32 bb = bk[it];
                u32 pos = loff[bb] + atomicAdd(&fill[bb], 1u);
                sval[pos] = v[it];
                sbkt[pos] = (unsigned char)bb;
            }
        }
        __syncthreads();
        for (u32 p = tid; p < clen; p += EXCP_THREADS) {
            u32 bb = sbkt[p];
            part[(u64)goff[bb] + (p - loff[bb])] = sval[p];
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------- P4: exact totals per bucket
// One wave per (stream, bucket): exact signed sum, minimum and maximum key.
__global__ __launch_bounds__(EXCP_THREADS) void k_km_bucket_stats(Workspace w, GroupParams g) {
    __shared__ u64 bins[4][EXCP_ABSM_BINS];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 nseg = 3u * g.ntensors;
    const u64 gw = (u64)blockIdx.x * 4 + wave;
    if (gw >= (u64)nseg * NBKT) return;
    const u32 sidx = (u32)(gw / NBKT), b = (u32)(gw % NBKT);
    if (w.seg[sidx].len == 0) return;
    const u32 *begin = w.km_begin + (u64)sidx * (NBKT + 1);
    const u32 p0 = begin[b], p1 = begin[b + 1];
    u64 *out = w.km_bsum + ((u64)sidx * NBKT + b) * EXCP_ABSM_BINS;
    if (lane < EXCP_ABSM_BINS) bins[wave][lane] = 0;
    u32 kmin = 0xffffffffu, kmax = 0;
    const float *__restrict__ part = seg_part(w, sidx);
    u64 *mybins = bins[wave];
    auto add = [&](u32 bin, u64 d) { atomicAdd(&mybins[bin], d); };
    for (u32 p = p0; p < p1; p += 64 * 8) {
        float x[8]; bool sel[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            u32 i = p + j * 64 + lane;
            sel[j] = i < p1;
            x[j] = sel[j] ? part[i] : 0.f;
            if (sel[j]) { u32 k = key_of(x[j]); kmin = min(kmin, k); kmax = max(kmax, k); }
        }
        wave_exact_add<8>(x, sel, add);
    }
#pragma unroll
    for (int mm = 32; mm >= 1; mm >>= 1) {
        kmin = min(kmin, (u32)__shfl_xor(kmin, mm, WAVE));
        kmax = max(kmax, (u32)__shfl_xor(kmax, mm, WAVE));
    }
    if (lane < EXCP_ABSM_BINS) out[lane] = bins[wave][lane];
    if (lane == 0) { w.km_min[(u64)sidx * NBKT + b] = kmin; w.km_max[(u64)sidx * NBKT + b] = kmax; }
}

// ---------------------------------------------------------------- P6: initial centres
// One workgroup per (stream, rank): radix select inside the bucket that holds the rank; the bits
// that the bucket's minimum and maximum key share are known and skipped.
__global__ __launch_bounds__(EXCP_THREADS) void k_km_init(Workspace w, GroupParams g) {
    __shared__ u32 hist[256];
    __shared__ u32 s_pick[2];
    const u32 K = (u32)g.K;
    const u32 sidx = blockIdx.x / K, k = blockIdx.x % K, tid = threadIdx.x;
    SegState &S = w.seg[sidx];
    const u64 len = S.len;
    if (len == 0) { if (tid == 0) S.C[k] = 0.f; return; }
    const u32 *begin = w.km_begin + (u64)sidx * (NBKT + 1);
    const u32 r = (u32)(((u64)(2 * k + 1) * len) / (2ull * K));
    u32 lo = 0, hi = NBKT;                  // begin[lo] <= r < begin[hi]
    while (hi - lo > 1) { u32 mid = (lo + hi) >> 1; if (begin[mid] <= r) lo = mid; else hi = mid; }
    const u32 b = lo, p0 = begin[b], p1 = begin[b + 1];
    u32 rank = r - p0;
    const u32 kmin = w.km_min[(u64)sidx * NBKT + b], kmax = w.km_max[(u64)sidx * NBKT + b];
    const float *__restrict__ part = seg_part(w, sidx);
    u32 diff = kmin ^ kmax;
    if (diff == 0) { if (tid == 0) S.C[k] = val_of(kmin); return; }
    int hb = 31 - __clz((int)diff);          // highest bit in which keys of this bucket differ
    u32 prefix = kmin >> (hb + 1 > 31 ? 31 : hb + 1);
    if (hb == 31) prefix = 0;
    int top = hb;                            // bits [0, top] still unknown
    while (top >= 0) {
        const int width = top + 1 < 8 ? top + 1 : 8;
        const int shift = top + 1 - width;
        hist[tid] = 0;
        __syncthreads();
        for (u32 p = p0 + tid; p < p1; p += EXCP_THREADS) {
            u32 key = key_of(part[p]);
            bool match = (top == 31) ? true : ((key >> (top + 1)) == prefix);
            if (match) atomicAdd(&hist[(key >> shift) & ((1u << width) - 1u)], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            u32 rr = rank, bin = 0;
            const u32 nb = 1u << width;
            while (bin + 1 < nb && rr >= hist[bin]) { rr -= hist[bin]; ++bin; }
            s_pick[0] = bin; s_pick[1] = rr;
        }
        __syncthreads();
        prefix = (top == 31 && width == 32) ? s_pick[0] : ((prefix << width) | s_pick[0]);
        rank = s_pick[1];
        top = shift - 1;
        __syncthreads();
    }
    if (tid == 0) S.C[k] = val_of(prefix);
}

// ---------------------------------------------------------------- P5a: one Lloyd accumulation
// Classification (one workgroup per stream): every bucket is compared with the current centres.
// A bucket whose smallest and largest value go to the same centre adds its stored totals to that
// centre; a bucket that a cluster border cuts is split into work items of at most 8192 values.
struct KmItem { u32 sidx, p0, p1, range; };      // range = alo | ahi << 8

__global__ __launch_bounds__(EXCP_THREADS) void k_km_classify(Workspace w, GroupParams g) {
    __shared__ float s_C[EXCP_MAX_K + 1];
    __shared__ u32 s_scan[EXCP_THREADS];
    __shared__ u32 s_base;
    const u32 sidx = blockIdx.x, tid = threadIdx.x;
    const SegState &S = w.seg[sidx];
    if (S.len == 0) return;
    const int K = g.K;
    for (u32 k = tid; k < (u32)K; k += EXCP_THREADS) s_C[k] = S.C[k];
    __syncthreads();
    const u32 *begin = w.km_begin + (u64)sidx * (NBKT + 1);
    u64 *acc = w.km_acc + (u64)sidx * EXCP_MAX_K * (EXCP_ABSM_BINS + 1);     // [K][bins + count]
    const u32 b = tid;
    const u32 p0 = begin[b], p1 = begin[b + 1], cntb = p1 - p0;
    u32 alo = 0, ahi = 0;
    if (cntb) {
        alo = (u32)nearest_centre(val_of(w.km_min[(u64)sidx * NBKT + b]), s_C, K, nullptr);
        ahi = (u32)nearest_centre(val_of(w.km_max[(u64)sidx * NBKT + b]), s_C, K, nullptr);
    }
    const bool cut = cntb && alo != ahi;
    if (cntb && !cut) {
        u64 *dst = acc + (u64)alo * (EXCP_ABSM_BINS + 1);
        const u64 *src = w.km_bsum + ((u64)sidx * NBKT + b) * EXCP_ABSM_BINS;
        for (int q = 0; q < EXCP_ABSM_BINS; ++q) { u64 v = src[q]; if (v) atomicAdd(&dst[q], v); }
        atomicAdd(&dst[EXCP_ABSM_BINS], (u64)cntb);
    }
    const u32 nitems = cut ? (cntb + EXCP_CHUNK - 1) / EXCP_CHUNK : 0u;
    s_scan[tid] = nitems;
    __syncthreads();
    for (u32 off = 1; off < EXCP_THREADS; off <<= 1) {
        u32 v = (tid >= off) ? s_scan[tid - off] : 0u;
        __syncthreads();
        s_scan[tid] += v;
        __syncthreads();
    }
    if (tid == EXCP_THREADS - 1) s_base = s_scan[tid] ? atomicAdd(w.km_item_count, s_scan[tid]) : 0u;
    __syncthreads();
    u32 at = s_base + s_scan[tid] - nitems;
    KmItem *items = (KmItem *)w.km_items;
    for (u32 q = 0; q < nitems; ++q, ++at) {
        if (at >= w.km_item_cap) { atomicExch(w.err_flag, 1); break; }
        u32 a0 = p0 + q * EXCP_CHUNK, a1 = a0 + EXCP_CHUNK < p1 ? a0 + EXCP_CHUNK : p1;
        items[at] = KmItem{sidx, a0, a1, alo | (ahi << 8)};
    }
}

// Work items: the values of a cut bucket are assigned one by one and added, exactly, to their
// centres.  Sums are gathered in LDS per item and flushed with a few integer atomics.
constexpr u32 ITEM_R = 8;      // centres per item held in LDS; wider ranges go straight to global memory

__global__ __launch_bounds__(EXCP_THREADS) void k_km_iter(Workspace w, GroupParams g) {
    __shared__ float s_C[EXCP_MAX_K + 1];
    __shared__ u64 s_bins[ITEM_R][EXCP_ABSM_BINS + 1];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int K = g.K;
    u32 nitems = *w.km_item_count;
    if (nitems > w.km_item_cap) nitems = w.km_item_cap;
    const KmItem *items = (const KmItem *)w.km_items;
    u32 cur = 0xffffffffu;
    for (u32 it = blockIdx.x; it < nitems; it += gridDim.x) {
        const KmItem I = items[it];
        __syncthreads();
        if (I.sidx != cur) {
            for (u32 k = tid; k < (u32)K; k += EXCP_THREADS) s_C[k] = w.seg[I.sidx].C[k];
            cur = I.sidx;
        }
        for (u32 i = tid; i < ITEM_R * (EXCP_ABSM_BINS + 1); i += EXCP_THREADS) (&s_bins[0][0])[i] = 0;
        __syncthreads();
        const u32 c_lo = I.range & 255u, c_hi = I.range >> 8;
        const bool in_lds = (c_hi - c_lo) < ITEM_R;
        u64 *acc = w.km_acc + (u64)I.sidx * EXCP_MAX_K * (EXCP_ABSM_BINS + 1);
        const float *__restrict__ part = seg_part(w, I.sidx);
        for (u32 p = I.p0 + wave * 512; p < I.p1; p += 4 * 512) {
            float x[8]; bool ok[8]; u32 a[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                u32 i = p + j * 64 + lane;
                ok[j] = i < I.p1;
                x[j] = ok[j] ? part[i] : 0.f;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = ok[j] ? (u32)nearest_centre(x[j], s_C, K, nullptr) : 0xffffffffu;
            for (u32 cl = c_lo; cl <= c_hi; ++cl) {
                bool sel[8]; u32 n = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) { sel[j] = a[j] == cl; n += __popcll(ballot64(sel[j])); }
                if (n == 0) continue;
                if (in_lds) {
                    u64 *dst = s_bins[cl - c_lo];
                    auto add = [&](u32 bin, u64 d) { atomicAdd(&dst[bin], d); };
                    wave_exact_add<8>(x, sel, add);
                    if (lane == 0) atomicAdd(&dst[EXCP_ABSM_BINS], (u64)n);
                } else {
                    u64 *dst = acc + (u64)cl * (EXCP_ABSM_BINS + 1);
                    auto add = [&](u32 bin, u64 d) { atomicAdd(&dst[bin], d); };
                    wave_exact_add<8>(x, sel, add);
                    if (lane == 0) atomicAdd(&dst[EXCP_ABSM_BINS], (u64)n);
                }
            }
        }
        __syncthreads();
        if (in_lds) {
            for (u32 i = tid; i < ITEM_R * (EXCP_ABSM_BINS + 1); i += EXCP_THREADS) {
                u64 v = (&s_bins[0][0])[i];
                u32 cl = c_lo + i / (EXCP_ABSM_BINS + 1);
                if (v && cl <= c_hi) atomicAdd(&acc[(u64)cl * (EXCP_ABSM_BINS + 1) + i % (EXCP_ABSM_BINS + 1)], v);
            }
        }
    }
}

// ---------------------------------------------------------------- P5b: move the centres
__global__ __launch_bounds__(EXCP_THREADS) void k_km_update(Workspace w, GroupParams g) {
    const u32 sidx = blockIdx.x, tid = threadIdx.x;
    SegState &S = w.seg[sidx];
    if (sidx == 0 && tid == 0) *w.km_item_count = 0;       // the work list is rebuilt every iteration
    if (S.len == 0) return;
    const u32 K = (u32)g.K;
    u64 *acc = w.km_acc + (u64)sidx * EXCP_MAX_K * (EXCP_ABSM_BINS + 1);
    for (u32 k = tid; k < K; k += EXCP_THREADS) {
        u64 *a = acc + (u64)k * (EXCP_ABSM_BINS + 1);
        const u64 cnt = a[EXCP_ABSM_BINS];
        if (cnt) {
            double sum = signed_bins_to_double(a);
            S.C[k] = (float)(sum / (double)cnt);
        }
        for (int q = 0; q <= EXCP_ABSM_BINS; ++q) a[q] = 0;
    }
}

// ---------------------------------------------------------------- final assignment + packing
// A chunk's codes are staged as bytes in LDS, then each thread assembles whole 64-bit words.
__global__ __launch_bounds__(EXCP_THREADS) void k_assign_pack(Workspace w, GroupParams g) {
    __shared__ float s_C[EXCP_MAX_K + 1];
    __shared__ unsigned char s_code[EXCP_CHUNK + 64];
    __shared__ double s_red[EXCP_THREADS / 64];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 total = *w.chunk_total;
    const u32 G = gridDim.x, b = blockIdx.x;
    const u32 lo = (u32)(((u64)b * total) / G), hi = (u32)(((u64)(b + 1) * total) / G);
    if (lo >= hi) return;
    const u32 nseg = 3u * g.ntensors;
    const int K = g.K;
    const u32 nbits = (u32)g.nbits;
    const u32 words_per_chunk = EXCP_CHUNK * nbits / 64u;

    u32 sidx = 0xffffffffu, s_end = 0;
    for (u32 c = lo; c < hi; ++c) {
        if (sidx == 0xffffffffu || c >= s_end) {
            __syncthreads();
            sidx = find_owner(w.seg_chunk_begin, nseg, c);
            s_end = w.seg_chunk_begin[sidx + 1];
            for (u32 k = tid; k < (u32)K; k += EXCP_THREADS) s_C[k] = w.seg[sidx].C[k];
            __syncthreads();
        }
        const SegState &S = w.seg[sidx];
        const u32 t = sidx / 3u, which = sidx % 3u;
        const TState &T = w.st[t];
        const float *__restrict__ x = seg_data(w, sidx);
        const u64 len = S.len;
        const u64 ebase = (u64)(c - S.chunk_begin) * EXCP_CHUNK;
        const u32 clen = (len - ebase) < EXCP_CHUNK ? (u32)(len - ebase) : EXCP_CHUNK;
        const u64 nwords = excp_words(len * nbits);
        u64 *out = (u64 *)(w.desc[t].blob + (which == 0 ? T.off_cw : (which == 1 ? T.off_cm : T.off_cv)));
        const u64 wbase = (u64)(c - S.chunk_begin) * words_per_chunk;
        double obj = 0.0;
        float v[PER_THREAD];
#pragma unroll
        for (u32 it = 0; it < PER_THREAD; ++it) {
            u32 e = it * EXCP_THREADS + tid;
            v[it] = (e < clen) ? x[ebase + e] : 0.f;
        }
#pragma unroll
        for (u32 it = 0; it < PER_THREAD; ++it) {
            u32 e = it * EXCP_THREADS + tid;
            u32 code = 0;
            if (e < clen) {
                double dist;
                code = 1u + (u32)nearest_centre(v[it], s_C, K, &dist);
                obj += dist;
            }
            s_code[e] = (unsigned char)code;
        }
        if (tid < 64) s_code[EXCP_CHUNK + tid] = 0;
        __syncthreads();
        for (u32 wl = tid; wl < words_per_chunk; wl += EXCP_THREADS) {
            const u64 wg = wbase + wl;
            if (wg >= nwords) break;
            const u32 bit0 = wl * 64u;
            u32 e = bit0 / nbits;
            int sh = (int)(e * nbits) - (int)bit0;          // <= 0 for the first code of the word
            u64 word = 0;
            while (sh < 64) {
                u64 code = s_code[e];
                word |= (sh >= 0) ? (code << sh) : (code >> (-sh));
                ++e; sh += (int)nbits;
            }
            out[wg] = word;
            if (wg == nwords - 1 && (nwords & 1ull)) out[nwords] = 0ull;     // 16-byte padding
        }
#pragma unroll
        for (int mm = 32; mm >= 1; mm >>= 1) obj += shfl_xor_f64(obj, mm);
        if (lane == 0) s_red[wave] = obj;
        __syncthreads();
        if (tid == 0) w.part_obj[c] = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
        __syncthreads();
    }
}

// ---------------------------------------------------------------- header, codebooks, results
__global__ __launch_bounds__(EXCP_THREADS) void k_finalize(Workspace w, GroupParams g, u32 rec_base) {
    __shared__ double s_obj[3];
    const u32 t = blockIdx.x, tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const TDesc &D = w.desc[t];
    TState &T = w.st[t];
    const u32 E = 1u << g.nbits;
    if (wave < 3) {
        const u32 sidx = 3u * t + wave;
        double acc = 0.0;
        if (w.seg[sidx].len) {
            const u32 c0 = w.seg[sidx].chunk_begin, c1 = w.seg_chunk_begin[sidx + 1];
            for (u32 c = c0 + lane; c < c1; c += 64) acc += w.part_obj[c];
        }
#pragma unroll
        for (int mm = 32; mm >= 1; mm >>= 1) acc += shfl_xor_f64(acc, mm);
        if (lane == 0) s_obj[wave] = acc;
    }
    __syncthreads();
    // codebooks: entry 0 is +0, then the K centres
    float *books = (float *)(D.blob + EXCP_HEADER);
    for (u32 i = tid; i < 3u * E; i += EXCP_THREADS) {
        u32 which = i / E, e = i % E;
        books[i] = (e == 0) ? 0.f : w.seg[3u * t + which].C[e - 1];
    }
    if (tid == 0) {
        int status = T.status;
        if (*w.err_flag) status = -7;
        T.obj[0] = s_obj[0]; T.obj[1] = s_obj[1]; T.obj[2] = s_obj[2];
        u32 *h = (u32 *)D.blob;
        u64 *h64 = (u64 *)D.blob;
        float *hf = (float *)D.blob;
        h[0] = EXCP_MAGIC; h[1] = EXCP_VERSION; h[2] = (u32)g.nbits; h[3] = g.flags;
        h64[2] = D.n; h64[3] = T.n_w; h64[4] = T.n_o;
        hf[10] = g.alpha; hf[11] = g.beta; hf[12] = u2f(T.med_bits); hf[13] = T.mean32;
        hf[14] = T.t_w; hf[15] = T.r_o;
        h64[8] = T.blob_bytes;
        h[18] = (u32)g.iters; h[19] = 0u;
        HostRec &R = w.rec_dev[rec_base + t];
        R.n = D.n; R.n_w = T.n_w; R.n_o = T.n_o; R.blob_bytes = T.blob_bytes; R.nonfinite = T.nonfinite;
        R.abs_sum = T.abs_sum; R.obj[0] = s_obj[0]; R.obj[1] = s_obj[1]; R.obj[2] = s_obj[2];
        R.med = u2f(T.med_bits); R.mean32 = T.mean32; R.t_w = T.t_w; R.r_o = T.r_o;
        R.status = status; R.pad = 0;
    }
}

}  // namespace

void launch_km_partition(const Workspace &w, const GroupParams &g, int phase, hipStream_t s) {
    if (!g.ntensors) return;
    const u32 nseg = 3 * g.ntensors;
    switch (phase) {
        case 0: hipLaunchKernelGGL(k_km_sample, dim3(nseg), dim3(EXCP_THREADS), 0, s, w, g); break;
        case 1: hipLaunchKernelGGL(k_km_count, dim3(w.grid_stream), dim3(EXCP_THREADS), 0, s, w, g); break;
        case 2: hipLaunchKernelGGL(k_km_scan, dim3(nseg), dim3(1024), 0, s, w, g); break;
        case 3: hipLaunchKernelGGL(k_km_scatter, dim3(w.grid_stream), dim3(EXCP_THREADS), 0, s, w, g); break;
        case 4: hipLaunchKernelGGL(k_km_bucket_stats, dim3(nseg * (NBKT / 4)), dim3(EXCP_THREADS), 0, s, w, g); break;
        default: break;
    }
}

void launch_km_init(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_km_init, dim3(3 * g.ntensors * (u32)g.K), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_km_classify(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_km_classify, dim3(3 * g.ntensors), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_km_iter(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_km_iter, dim3(w.grid_stream), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_km_update(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_km_update, dim3(3 * g.ntensors), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_assign_pack(const Workspace &w, const GroupParams &g, hipStream_t s) {
    hipLaunchKernelGGL(k_assign_pack, dim3(w.grid_stream), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_finalize(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_finalize, dim3(g.ntensors), dim3(EXCP_THREADS), 0, s, w, g, w.rec_base);
}
