// Full-tensor statistics for the pruning thresholds of Sec. 3.2:
//   * the lower median of |W_t - W_prev| per tensor (Eq. "r_w") by a three-pass radix-histogram
//     select over the 31-bit magnitude keys (11 + 11 + 9 bits), histograms held in LDS;
//   * the exact sum of |m| per tensor (Eq. "r_o") by integer accumulation: every |m_i| is
//     mant * 2^(pos-149); a wave adds its mantissas in a 40-bit exponent window as integers and
//     files the result into per-tensor u64 bins 8 binary orders apart, so the sum is exact and
//     does not depend on the order of additions;
//   * non-finite detection on W_prev, W_t, m and the residual.
#include "excp_util.h"

namespace {

template <int PASS>
__global__ __launch_bounds__(EXCP_THREADS) void k_stats_hist(Workspace w, GroupParams g) {
    constexpr int NB = (PASS == 2) ? 512 : 2048;
    __shared__ u32 hist[NB];
    __shared__ u64 bins[EXCP_ABSM_BINS];
    __shared__ u32 s_nf;
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 G = gridDim.x, b = blockIdx.x;
    const u32 lo = (u32)(((u64)b * g.ntiles) / G), hi = (u32)(((u64)(b + 1) * g.ntiles) / G);
    if (lo >= hi) return;

    for (u32 i = tid; i < NB; i += EXCP_THREADS) hist[i] = 0;
    if (tid < EXCP_ABSM_BINS) bins[tid] = 0;
    if (tid == 0) s_nf = 0;
    __syncthreads();

    u32 t = find_owner(w.tile_begin, g.ntensors, lo);
    u32 t_end = w.tile_begin[t + 1];
    u32 nf = 0;

    auto flush = [&](u32 tt) {
        __syncthreads();
        for (u32 i = tid; i < NB; i += EXCP_THREADS) {
            u32 c = hist[i];
            if (c) { atomicAdd(&w.med_hist[(u64)tt * 2048u + i], c); hist[i] = 0; }
        }
        if (PASS == 0) {
            if (tid < EXCP_ABSM_BINS) {
                u64 c = bins[tid];
                if (c) { atomicAdd(&w.st[tt].absm[tid], c); bins[tid] = 0; }
            }
            if (nf) atomicAdd(&s_nf, nf);
            nf = 0;
            __syncthreads();
            if (tid == 0 && s_nf) { atomicAdd(&w.st[tt].nonfinite, (u64)s_nf); s_nf = 0; }
        }
        __syncthreads();
    };

    for (u32 tile = lo; tile < hi; ++tile) {
        if (tile >= t_end) {
            flush(t);
            t = find_owner(w.tile_begin, g.ntensors, tile);
            t_end = w.tile_begin[t + 1];
        }
        const TDesc &D = w.desc[t];
        const u64 n = D.n;
        const u64 base = (u64)(tile - D.tile_begin) * EXCP_TILE;
        const float *__restrict__ Wp = D.Wp, *__restrict__ W = D.W, *__restrict__ M = D.m;
        u32 prefix = 0;
        if (PASS > 0) prefix = w.st[t].sel_prefix;

        u32 key[16];
        u32 mb[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            u64 idx = base + (u64)((wave * 16 + j) * 64 + lane);
            bool ok = idx < n;
            float a = ok ? W[idx] : 0.f;
            float p = ok ? Wp[idx] : 0.f;
            float d = a - p;
            u32 k = f2u(d) & 0x7fffffffu;
            key[j] = ok ? k : 0xffffffffu;
            if (PASS == 0) {
                float mm = ok ? M[idx] : 0.f;
                mb[j] = f2u(mm) & 0x7fffffffu;
                u32 bad = ((f2u(a) & 0x7f800000u) == 0x7f800000u) || ((f2u(p) & 0x7f800000u) == 0x7f800000u) ||
                          ((mb[j] & 0x7f800000u) == 0x7f800000u) || ((k & 0x7f800000u) == 0x7f800000u);
                nf += bad;
                if (bad) mb[j] = 0;
            }
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            u32 k = key[j];
            if (k != 0xffffffffu) {
                if (PASS == 0) atomicAdd(&hist[k >> 20], 1u);
                if (PASS == 1) { if ((k >> 20) == prefix) atomicAdd(&hist[(k >> 9) & 2047u], 1u); }
                if (PASS == 2) { if ((k >> 9) == prefix) atomicAdd(&hist[k & 511u], 1u); }
            }
        }
        if (PASS == 0) {
            // exact sum of |m| for this wave's 1024 values
            u32 pmax = 0;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                u32 e = mb[j] >> 23;
                u32 pos = (e ? e : 1u) - 1u;
                if (mb[j]) pmax = max(pmax, pos);
            }
            pmax = wave_max_u32(pmax);
            const u32 B = pmax > 39u ? pmax - 39u : 0u;
            u64 accL = 0, accH = 0;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                u32 e = mb[j] >> 23;
                u32 mant = (mb[j] & 0x7fffffu) | (e ? 0x800000u : 0u);
                u32 pos = (e ? e : 1u) - 1u;
                if (mant) {
                    if (pos >= B) {
                        u64 term = (u64)mant << (pos - B);
                        accL += term & 0xffffffffull;
                        accH += term >> 32;
                    } else {
                        atomicAdd(&bins[pos >> 3], (u64)mant << (pos & 7u));
                    }
                }
            }
            accL = wave_sum_u64(accL);
            accH = wave_sum_u64(accH);
            if (lane == 0) {
                u64 lo64 = accL + (accH << 32);
                u64 hi64 = (accH >> 32) + (lo64 < accL ? 1ull : 0ull);
                u64 piece[3] = {lo64 & 0xffffffffull, lo64 >> 32, hi64};
#pragma unroll
                for (int q = 0; q < 3; ++q) {
                    u32 p = B + 32u * q;
                    if (piece[q]) atomicAdd(&bins[p >> 3], piece[q] << (p & 7u));
                }
            }
            // clear this tile's share of the bitmap_o region (filled later with atomic ORs)
            if (tid < 66) {
                u64 word = (base >> 6) + tid;
                u64 nw = excp_words(n) + 2;
                u64 off = EXCP_HEADER + 12ull * (1u << g.nbits) + excp_pad16(8ull * excp_words(n)) + 8ull * word;
                if (tid < 64 ? (word < nw) : (base + EXCP_TILE >= n && word < nw))
                    if (off + 8 <= D.blob_cap) *(u64 *)(D.blob + off) = 0ull;
            }
        }
    }
    flush(t);
}

// Exact sum: bins[g] * 2^(8g-149) summed as one big integer, rounded once (to nearest, ties to
// even) to fp64.
__device__ double absm_bins_to_double(const u64 *bins) {
    u32 limb[14];
    for (int i = 0; i < 14; ++i) limb[i] = 0;
    for (int gidx = 0; gidx < EXCP_ABSM_BINS; ++gidx) {
        u64 c = bins[gidx];
        if (!c) continue;
        u32 bit = 8u * gidx, li = bit >> 5, sh = bit & 31u;
        // c << sh spans up to three limbs
        u64 lo = c << sh;
        u32 top = sh ? (u32)(c >> (64 - sh)) : 0u;
        u32 parts[3] = {(u32)lo, (u32)(lo >> 32), top};
        u64 carry = 0;
        for (int q = 0; q < 3 || carry; ++q) {
            if (li + q >= 14) break;
            u64 s = (u64)limb[li + q] + (q < 3 ? parts[q] : 0u) + carry;
            limb[li + q] = (u32)s;
            carry = s >> 32;
        }
    }
    int top = -1;
    for (int i = 13; i >= 0; --i) if (limb[i]) { top = i; break; }
    if (top < 0) return 0.0;
    int msb = 32 * top + (31 - __clz((int)limb[top]));       // position of the leading one
    auto bit_at = [&](int p) -> u32 { return p < 0 ? 0u : (limb[p >> 5] >> (p & 31)) & 1u; };
    if (msb <= 52) {
        u64 x = (u64)limb[0] | ((u64)limb[1] << 32);
        return ldexp((double)x, -149);
    }
    u64 mant = 0;
    for (int p = msb; p >= msb - 52; --p) mant = (mant << 1) | bit_at(p);
    u32 guard = bit_at(msb - 53);
    u32 sticky = 0;
    for (int p = msb - 54; p >= 0 && !sticky; --p) sticky |= bit_at(p);
    if (guard && (sticky || (mant & 1ull))) mant += 1;       // 2^53 is still exact in fp64
    return ldexp((double)mant, msb - 52 - 149);
}

template <int PASS>
__global__ __launch_bounds__(EXCP_THREADS) void k_median_resolve(Workspace w, GroupParams g) {
    constexpr int NB = (PASS == 2) ? 512 : 2048;
    constexpr int PER = NB / EXCP_THREADS;
    __shared__ u32 s_sum[EXCP_THREADS];
    const u32 t = blockIdx.x, tid = threadIdx.x;
    const u64 n = w.desc[t].n;
    TState &S = w.st[t];
    u32 *H = w.med_hist + (u64)t * 2048u;
    if (n == 0) {
        if (tid == 0 && PASS == 2) { S.med_bits = 0; S.mean32 = 0.f; S.t_w = 0.f; S.r_o = 0.f; S.abs_sum = 0.0; }
        return;
    }
    u32 rank = (PASS == 0) ? (u32)((n - 1) >> 1) : S.sel_rank;
    u32 prefix = (PASS == 0) ? 0u : S.sel_prefix;
    u32 c[PER], local = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) { c[i] = H[tid * PER + i]; local += c[i]; H[tid * PER + i] = 0; }
    s_sum[tid] = local;
    __syncthreads();
    // exclusive prefix of the per-thread sums (256 values; a plain doubling scan)
    for (int off = 1; off < EXCP_THREADS; off <<= 1) {
        u32 v = (tid >= (u32)off) ? s_sum[tid - off] : 0u;
        __syncthreads();
        s_sum[tid] += v;
        __syncthreads();
    }
    u32 before = s_sum[tid] - local;
    if (rank >= before && rank < before + local) {           // exactly one thread
        u32 r = rank - before;
        int i = 0;
        while (r >= c[i]) { r -= c[i]; ++i; }
        u32 bin = tid * PER + i;
        u32 np = (PASS == 2) ? ((prefix << 9) | bin) : ((prefix << 11) | bin);
        S.sel_prefix = np;
        S.sel_rank = r;
        if (PASS == 2) {
            S.med_bits = np;
            float med = u2f(np);
            S.t_w = __fmul_rn(g.alpha, med);
            double sum = absm_bins_to_double(S.absm);
            double mean64 = sum / (double)n;
            float mean32 = (float)mean64;
            S.abs_sum = sum;
            S.mean32 = mean32;
            S.r_o = __fmul_rn(g.beta, mean32);
        }
    }
}

__global__ void k_zero_u32(u32 *p, u64 count) {
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    u64 stride = (u64)gridDim.x * blockDim.x;
    for (; i < count; i += stride) p[i] = 0u;
}

}  // namespace

void launch_zero_u32(u32 *p, u64 count, hipStream_t s) {
    if (!count) return;
    u64 blocks = (count + 1023) / 1024;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_zero_u32, dim3((u32)blocks), dim3(256), 0, s, p, count);
}

void launch_stats_hist(const Workspace &w, const GroupParams &g, int pass, hipStream_t s) {
    if (!g.ntiles) return;
    dim3 grid(w.grid_stream), block(EXCP_THREADS);
    if (pass == 0) hipLaunchKernelGGL(k_stats_hist<0>, grid, block, 0, s, w, g);
    else if (pass == 1) hipLaunchKernelGGL(k_stats_hist<1>, grid, block, 0, s, w, g);
    else hipLaunchKernelGGL(k_stats_hist<2>, grid, block, 0, s, w, g);
}

void launch_median_resolve(const Workspace &w, const GroupParams &g, int pass, hipStream_t s) {
    if (!g.ntensors) return;
    dim3 grid(g.ntensors), block(EXCP_THREADS);
    if (pass == 0) hipLaunchKernelGGL(k_median_resolve<0>, grid, block, 0, s, w, g);
    else if (pass == 1) hipLaunchKernelGGL(k_median_resolve<1>, grid, block, 0, s, w, g);
    else hipLaunchKernelGGL(k_median_resolve<2>, grid, block, 0, s, w, g);
}
