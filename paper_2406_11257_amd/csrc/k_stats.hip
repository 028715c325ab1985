// Full-tensor statistics for the pruning thresholds of Sec. 3.2:
//   * the lower median of |W_t - W_prev| per tensor (Eq. "r_w"), exactly, in ONE pass over the
//     tensor: a sorted sample of 8192 residuals brackets the median between two keys lo <= hi; the
//     streaming pass counts the keys below lo and collects the few per cent of keys inside the
//     bracket; a radix-histogram select (LDS histograms, 11 bits per pass) over those candidates
//     then finds the order statistic.  The bracket can miss (probability about 2e-5 per tensor, or
//     adversarial data); the counts reveal that, and the tensor then takes the always-correct
//     fallback: a three-pass radix-histogram select over the whole tensor (11 + 11 + 9 key bits);
//   * the exact sum of |m| per tensor (Eq. "r_o") by integer accumulation: every |m_i| is
//     mant * 2^(pos-149).  The sample fixes a window of 24 bit positions per tensor that holds
//     practically every value; inside it a value is a multiple of one unit below 2^48 units, so a
//     lane adds sixteen of them exactly in fp64, splits the sum into two 32-bit integers and keeps
//     those in 64-bit counters; values outside the window (rare) are filed one by one.  Everything
//     ends in per-tensor u64 bins 8 binary orders apart, so the sum is exact and does not depend on
//     the order of additions;
//   * non-finite detection on W_prev, W_t, m and the residual.
#include "excp_util.h"

namespace {

constexpr u32 MED_SAMPLE = 8192;      // sample size (and the size up to which a tensor is simply sorted)
constexpr u32 MED_HALF_WIDTH = 192;   // bracket = sample ranks 4096 -+ 192 (about 4.2 sigma of the sample rank)
constexpr u32 CAND_PER_WAVE = 1024;
constexpr u32 MED_THREADS = 1024;     // workgroup of the sampling kernel: one per tensor, so its own latency is the kernel's

enum { MED_PENDING = 0, MED_KNOWN = 1, MED_FALLBACK = 2 };

__device__ __forceinline__ void sort_keys_lds(u32 *key, u32 count_pow2) {
    const u32 tid = threadIdx.x;
    for (u32 k = 2; k <= count_pow2; k <<= 1) {
        for (u32 j = k >> 1; j > 0; j >>= 1) {
            for (u32 t = tid; t < count_pow2 / 2; t += MED_THREADS) {
                u32 i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                u32 p = i | j;
                u32 a = key[i], b = key[p];
                bool asc = (i & k) == 0;
                if ((a > b) == asc) { key[i] = b; key[p] = a; }
            }
            __syncthreads();
        }
    }
}

// One workgroup per tensor: sample (or all) residual magnitudes, sorted.
__global__ __launch_bounds__(MED_THREADS) void k_median_sample(Workspace w, GroupParams g) {
    __shared__ u32 key[MED_SAMPLE];
    __shared__ u32 s_mmax;
    const u32 t = blockIdx.x, tid = threadIdx.x;
    const TDesc &D = w.desc[t];
    TState &S = w.st[t];
    const u64 n = D.n;
    if (n == 0) { if (tid == 0) { S.med_bits = 0; S.med_state = MED_KNOWN; } return; }
    if (tid == 0) s_mmax = 0;
    __syncthreads();
    const u32 ns = n < MED_SAMPLE ? (u32)n : MED_SAMPLE;
    u32 mmax = 0;                                   // largest finite |m| pattern of the sample
#pragma unroll
    for (u32 i = tid; i < MED_SAMPLE; i += MED_THREADS) {       // eight samples per thread, their loads side by side
        u32 k = 0xffffffffu;
        if (i < ns) {
            const u64 idx = n <= MED_SAMPLE ? (u64)i : ((u64)i * n) / MED_SAMPLE;
            const u32 wt = excp_wtype(g.flags);
            const float wv = load_weight(D.W, idx, wt);
            k = f2u((g.flags & 1u) ? wv : wv - load_weight(D.Wp, idx, wt)) & 0x7fffffffu;   // flag: median of |W_t|
            const u32 mb = f2u(D.m[idx]) & 0x7fffffffu;
            if (mb < 0x7f800000u) mmax = max(mmax, mb);
        }
        key[i] = k;
    }
    mmax = wave_max_u32(mmax);
    if ((tid & 63u) == 0) atomicMax(&s_mmax, mmax);
    __syncthreads();
    sort_keys_lds(key, MED_SAMPLE);
    if (tid == 0) {
        // window of the exact sum: its top sits 4 binary orders above the largest sampled |m|
        const u32 e = s_mmax >> 23;
        const u32 pos = (e ? e : 1u) - 1u;
        S.absm_base = pos + 4u > 23u ? min(pos + 4u - 23u, 230u) : 0u;
        if (n <= MED_SAMPLE) {
            S.med_bits = key[(n - 1) >> 1];
            S.med_state = MED_KNOWN;
        } else {
            const u32 a = MED_SAMPLE / 2 - MED_HALF_WIDTH, b = MED_SAMPLE / 2 + MED_HALF_WIDTH;
            S.br_lo = key[a];
            S.br_hi = key[b];
            S.med_state = MED_PENDING;
            // 16-bit weights: residuals are few distinct values.  Up to four values of the bracket
            // that fill at least 32 places of the sorted sample (0.4 % of the tensor) are counted
            // during the streaming pass instead of being listed one by one.
            u32 na = 0;
            if ((g.flags & 0x30u) && key[a] != key[b]) {
                for (u32 i = a; i <= b && na < 4u;) {
                    const u32 kv = key[i];
                    u32 j0 = i, j1 = i;
                    while (j0 > 0u && key[j0 - 1u] == kv) --j0;
                    while (j1 + 1u < MED_SAMPLE && key[j1 + 1u] == kv) ++j1;
                    if (j1 - j0 + 1u >= 32u) S.atom_key[na++] = kv;
                    i = j1 + 1u;
                }
            }
            S.natoms = na;
        }
    }
}

// Four consecutive floats at an address that is only known to be 4-byte aligned.
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

// The streaming pass: exact sum of |m|, non-finite check, count of keys below the bracket and
// collection of the keys inside it.  Persistent workgroups over contiguous tile ranges; a lane
// takes four consecutive elements of each of four 256-element rows of its wave's quarter tile.
// W16: the weights are 16-bit (fp16 or bf16 by the flags), four to an 8-byte load where the arrays
// allow it; they are widened on arrival and everything after that is the fp32 code.
template <bool W16>
__global__ __launch_bounds__(EXCP_THREADS) void k_stats_stream(Workspace w, GroupParams g) {
    __shared__ u64 bins[EXCP_ABSM_BINS];
    __shared__ u32 l_cand[4][2 * CAND_PER_WAVE + 1];   // per wave: staged candidates, plus a spare slot
    __shared__ u32 s_nf, s_lt;
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 G = gridDim.x, b = blockIdx.x;
    const u32 lo_tile = (u32)(((u64)b * g.ntiles) / G), hi_tile = (u32)(((u64)(b + 1) * g.ntiles) / G);
    if (lo_tile >= hi_tile) return;
    if (tid < EXCP_ABSM_BINS) bins[tid] = 0;
    if (tid == 0) { s_nf = 0; s_lt = 0; }
    __syncthreads();

    u32 t = find_owner(w.tile_begin, g.ntensors, lo_tile);
    u32 t_end = w.tile_begin[t + 1];
    u32 nf = 0, clt = 0;           // clt is the same in every lane of a wave
    u64 accL = 0, accH = 0;        // this lane's in-window units: sum of low / high 32-bit halves
    u32 B = w.st[t].absm_base;     // window = bit positions [B, B + 24)

    u32 acnt[4] = {0u, 0u, 0u, 0u};   // W16: elements equal to the tensor's counted bracket values (same in every lane)
    u32 wcount = 0;                // candidates this wave has staged in LDS (same in every lane)
    auto flush_cand = [&](u32 tt) {
        if (W16 && lane == 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q) if (acnt[q]) atomicAdd(&w.st[tt].atom_cnt[q], acnt[q]);
        }
        if (W16) { acnt[0] = acnt[1] = acnt[2] = acnt[3] = 0u; }
        // the staged candidates go to the tensor's list: one reservation for many tiles
        if (wcount) {
            const TDesc &D = w.desc[tt];
            const u32 L = D.cand_lists;
            const bool one_value = w.st[tt].br_lo == w.st[tt].br_hi;
            if (L == 1u) {
                u32 at = 0;
                if (lane == 0) at = atomicAdd(&w.st[tt].cand_count, wcount);
                at = __shfl(at, 0, WAVE);
                if (one_value) {
                    // a bracket of one value (heavily tied data, e.g. 16-bit weights that did not move):
                    // every candidate is that value, so their number is all that is needed
                } else if ((u64)at + wcount <= D.cand_cap) {
                    EXCP_GLOBAL u32 *dst = gptr(w.cand) + D.cand_off + at;
                    for (u32 i = lane; i < wcount; i += 64) dst[i] = l_cand[wave][i];
                } else if (lane == 0) {
                    atomicOr(&w.st[tt].cand_overflow, 1u);
                }
            } else {
                // a very large tensor: L lists with a counter each; a wave starts at "its" list and moves
                // on to the next when one is full, so the lists fail only when all of them are full
                u32 *ctr = w.cand_ctr + (u64)tt * 512u;
                const u32 cap = (u32)(D.cand_cap / L);
                u32 j = (blockIdx.x * 4u + wave) % L;
                bool placed = false;
                for (u32 attempt = 0; attempt < L && !placed; ++attempt, j = (j + 1u == L ? 0u : j + 1u)) {
                    u32 at = 0;
                    if (lane == 0) at = atomicAdd(&ctr[j * 32u], wcount);
                    at = __shfl(at, 0, WAVE);
                    if (one_value) { placed = true; break; }            // counted only
                    if ((u64)at + wcount <= cap) {
                        EXCP_GLOBAL u32 *dst = gptr(w.cand) + D.cand_off + (u64)j * cap + at;
                        for (u32 i = lane; i < wcount; i += 64) dst[i] = l_cand[wave][i];
                        if (lane == 0) atomicMax(&ctr[j * 32u + 1u], at + wcount);
                        placed = true;
                    }
                }
                if (!placed && lane == 0) atomicOr(&w.st[tt].cand_overflow, 1u);
            }
            wcount = 0;
        }
    };
    auto flush = [&](u32 tt) {
        flush_cand(tt);
        // the lanes' window sums, as three 32-bit pieces at positions B, B + 32, B + 64
        const u64 sumL = wave_sum_u64(accL), sumH = wave_sum_u64(accH);
        accL = 0; accH = 0;
        if (lane == 0) {
            const u64 lo64 = sumL + (sumH << 32);
            const u64 hi64 = (sumH >> 32) + (lo64 < sumL ? 1ull : 0ull);
            const u64 piece[3] = {lo64 & 0xffffffffull, lo64 >> 32, hi64};
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const u32 p = B + 32u * q;
                if (piece[q]) atomicAdd(&bins[p >> 3], piece[q] << (p & 7u));
            }
            if (clt) atomicAdd(&s_lt, clt);
        }
        if (nf) atomicAdd(&s_nf, nf);
        nf = 0; clt = 0;
        __syncthreads();
        if (tid < EXCP_ABSM_BINS) {
            u64 c = bins[tid];
            if (c) { atomicAdd(&w.st[tt].absm[tid], c); bins[tid] = 0; }
        }
        if (tid == 0) {
            if (s_nf) { atomicAdd(&w.st[tt].nonfinite, (u64)s_nf); s_nf = 0; }
            if (s_lt) { atomicAdd(&w.st[tt].c_lt, s_lt); s_lt = 0; }
        }
        __syncthreads();
    };

    for (u32 tile = lo_tile; tile < hi_tile; ++tile) {
        if (tile >= t_end) {
            flush(t);
            t = find_owner(w.tile_begin, g.ntensors, tile);
            t_end = w.tile_begin[t + 1];
            B = w.st[t].absm_base;
        }
        const TDesc &D = w.desc[t];
        TState &S = w.st[t];
        const u64 n = D.n;
        const u64 base = (u64)(tile - D.tile_begin) * EXCP_TILE;
        const u32 rem = (n - base < (u64)EXCP_TILE) ? (u32)(n - base) : EXCP_TILE;
        const bool pending = S.med_state == MED_PENDING;
        const u32 klo = S.br_lo, kspan = S.br_hi - klo;

        u32 key[16], mb[16];
        u32 worst = 0;             // largest magnitude pattern seen: >= 0x7f800000 means Inf or NaN
        const bool of_weights = (g.flags & 1u) != 0;       // the median is that of |W_t|, not of the residual
        {
            const EXCP_GLOBAL float *gW = gptr(D.W) + base, *gP = gptr(D.Wp) + base, *gM = gptr(D.m) + base;
            const u32 wt = W16 ? excp_wtype(g.flags) : 0u;
            const bool bf = wt == 2u;
            const EXCP_GLOBAL unsigned short *hW = gptr((const unsigned short *)D.W) + base;
            const EXCP_GLOBAL unsigned short *hP = gptr((const unsigned short *)D.Wp) + base;
            const bool vec16 = W16 && (((uintptr_t)D.W | (uintptr_t)D.Wp) & 7u) == 0u;   // 8-byte loads need 8-byte alignment
            if (rem == EXCP_TILE && (!W16 || vec16)) {
                f4u a[4], p[4], mm[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const u32 off = wave * 1024u + (u32)k * 256u + lane * 4u;
                    if (W16) {
                        const us4 ha = __builtin_nontemporal_load((const EXCP_GLOBAL us4 *)(hW + off));
                        const us4 hp = __builtin_nontemporal_load((const EXCP_GLOBAL us4 *)(hP + off));
#pragma unroll
                        for (int j = 0; j < 4; ++j) { a[k][j] = w16_widen(ha[j], bf); p[k][j] = w16_widen(hp[j], bf); }
                    } else {
                        a[k] = __builtin_nontemporal_load((const EXCP_GLOBAL f4u *)(gW + off));
                        p[k] = __builtin_nontemporal_load((const EXCP_GLOBAL f4u *)(gP + off));
                    }
                    mm[k] = __builtin_nontemporal_load((const EXCP_GLOBAL f4u *)(gM + off));
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float av = a[k][j], pv = p[k][j];
                        const u32 dk = f2u(av - pv) & 0x7fffffffu, wk = f2u(av) & 0x7fffffffu;
                        key[4 * k + j] = of_weights ? wk : dk;
                        mb[4 * k + j] = f2u(mm[k][j]) & 0x7fffffffu;
                        worst = max(max(worst, dk), max(mb[4 * k + j], max(wk, f2u(pv) & 0x7fffffffu)));
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const u32 off = wave * 1024u + (u32)(j >> 2) * 256u + lane * 4u + (u32)(j & 3);
                    const bool ok = off < rem;
                    float av = 0.f, pv = 0.f;
                    if (ok) {
                        av = W16 ? w16_widen(hW[off], bf) : gW[off];
                        pv = W16 ? w16_widen(hP[off], bf) : gP[off];
                    }
                    const float mv = ok ? gM[off] : 0.f;
                    const u32 dk = f2u(av - pv) & 0x7fffffffu, wk = f2u(av) & 0x7fffffffu;
                    mb[j] = f2u(mv) & 0x7fffffffu;
                    worst = max(max(worst, dk), max(mb[j], max(wk, f2u(pv) & 0x7fffffffu)));
                    key[j] = ok ? (of_weights ? wk : dk) : 0xffffffffu;      // above every bracket, never a candidate
                }
            }
        }
        if (__any(worst >= 0x7f800000u)) {
            // rare: something is not finite; it is reported and keeps out of the sum
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (key[j] != 0xffffffffu && (key[j] & 0x7f800000u) == 0x7f800000u) nf += 1;
                if ((mb[j] & 0x7f800000u) == 0x7f800000u) { nf += 1; mb[j] = 0; }
            }
            if (nf == 0 && worst >= 0x7f800000u) nf = 1;
        }
        const u32 natoms = W16 ? S.natoms : 0u;
        const u32 ak0 = S.atom_key[0], ak1 = S.atom_key[1], ak2 = S.atom_key[2], ak3 = S.atom_key[3];
        if (pending) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                clt += __popcll(ballot64(key[j] < klo));
                bool cand = key[j] - klo <= kspan;            // klo <= key <= khi (a padded key wraps far above)
                if (W16 && natoms) {
                    const bool e0 = key[j] == ak0, e1 = natoms > 1u && key[j] == ak1;
                    const bool e2 = natoms > 2u && key[j] == ak2, e3 = natoms > 3u && key[j] == ak3;
                    acnt[0] += __popcll(ballot64(e0)); acnt[1] += __popcll(ballot64(e1));
                    acnt[2] += __popcll(ballot64(e2)); acnt[3] += __popcll(ballot64(e3));
                    cand = cand && !(e0 || e1 || e2 || e3);
                }
                const u64 bal = ballot64(cand);
                // branch-free: the others write to a spare slot past the end
                const u32 below = __builtin_amdgcn_mbcnt_hi((u32)(bal >> 32), __builtin_amdgcn_mbcnt_lo((u32)bal, 0u));
                l_cand[wave][cand ? wcount + below : 2 * CAND_PER_WAVE] = key[j];
                wcount += __popcll(bal);
            }
            if (wcount > CAND_PER_WAVE) flush_cand(t);        // room for another 1024 is kept
        }
        {
            // exact sum of |m|: in-window values are whole multiples of 2^(B-149) below 2^48 units,
            // so this lane's sixteen add exactly in fp64.
            const u32 thr_lo = B ? ((B + 1u) << 23) : 0u, span = ((B + 25u) << 23) - thr_lo;
            double dsum = 0.0;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const bool in = mb[j] - thr_lo < span;
                dsum += in ? (double)u2f(mb[j]) : 0.0;
                if (!in && mb[j]) {
                    const u32 e = mb[j] >> 23;
                    const u32 mant = (mb[j] & 0x7fffffu) | (e ? 0x800000u : 0u);
                    const u32 pos = (e ? e : 1u) - 1u;
                    atomicAdd(&bins[pos >> 3], (u64)mant << (pos & 7u));
                }
            }
            const double units = ldexp(dsum, 149 - (int)B);                // an integer below 2^52
            const u32 hi32 = (u32)(units * 2.3283064365386963e-10);     // floor(units / 2^32)
            const u32 lo32 = (u32)(units - (double)hi32 * 4294967296.0);
            accL += lo32;
            accH += hi32;
        }
    }
    flush(t);
}

// After the streaming pass: does the bracket hold the median?  If so the select goes on inside
// the candidates (base key, number of undecided low bits, rank); if not the tensor falls back.
__global__ void k_cand_begin(Workspace w, GroupParams g) {
    const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= g.ntensors) return;
    TState &S = w.st[t];
    if (S.med_state != MED_PENDING) return;
    const u64 n = w.desc[t].n;
    const u64 r = (n - 1) >> 1;
    const u32 L = w.desc[t].cand_lists;
    u64 cnt = S.cand_count;
    if (L > 1u) {                          // several lists: slots asked for (counting only) or granted (listed)
        const u32 *ctr = w.cand_ctr + (u64)t * 512u;
        cnt = 0;
        for (u32 j = 0; j < L; ++j) cnt += ctr[j * 32u + (S.br_hi == S.br_lo ? 0u : 1u)];
        S.cand_count = (u32)cnt;
    }
    const u64 below = S.c_lt;
    if (S.br_hi == S.br_lo) {              // one-value bracket: only counted, never listed
        if (r >= below && r < below + cnt) { S.med_bits = S.br_lo; S.med_state = MED_KNOWN; }
        else S.med_state = MED_FALLBACK;
        return;
    }
    u64 counted = 0;                       // bracket values that were counted instead of listed
    for (u32 q = 0; q < S.natoms; ++q) counted += S.atom_cnt[q];
    if (S.cand_overflow || cnt > w.desc[t].cand_cap || r < below || r >= below + cnt + counted) {
        S.med_state = MED_FALLBACK;
        return;
    }
    const u32 span = S.br_hi - S.br_lo;
    S.sel_base = S.br_lo;
    S.sel_width = span ? 32u - (u32)__clz((int)span) : 0u;
    S.sel_rank = (u32)(r - below);
    if (span == 0) { S.med_bits = S.br_lo; S.med_state = MED_KNOWN; }
}

// One radix pass over the candidates: histogram of the top (up to 11) undecided bits.  A workgroup
// takes the candidates that belong to 256 consecutive tiles of the group's tile list -- for each
// tensor it meets, the matching share of that tensor's candidate list -- so that its LDS histogram
// is flushed once per tensor it meets and not once per tensor of the group.
constexpr u32 CAND_TILES = 256;

__global__ __launch_bounds__(EXCP_THREADS) void k_cand_hist(Workspace w, GroupParams g) {
    __shared__ u32 hist[2048];
    const u32 tid = threadIdx.x;
    const u32 lo = blockIdx.x * CAND_TILES, hi = min(lo + CAND_TILES, g.ntiles);
    if (lo >= hi) return;
    for (u32 i = tid; i < 2048; i += EXCP_THREADS) hist[i] = 0;
    __syncthreads();
    u32 t = find_owner(w.tile_begin, g.ntensors, lo);
    for (u32 a0 = lo; a0 < hi; ++t) {
        const u32 tb = w.tile_begin[t], te = w.tile_begin[t + 1];
        const u32 a1 = min(te, hi);                       // this workgroup's tiles of tensor t: [a0, a1)
        const TState &S = w.st[t];
        if (a1 > a0 && S.med_state == MED_PENDING && S.sel_width != 0) {
            const u32 base = S.sel_base, width = S.sel_width;
            const u32 shift = width > 11u ? width - 11u : 0u;
            const u64 limit = 1ull << width;
            const u32 tc = te - tb;
            const u32 L = w.desc[t].cand_lists, cap = (u32)(w.desc[t].cand_cap / L);
            auto tally = [&](u32 key) {
                const u32 rel = key - base;               // keys below base wrap around and drop out
                if ((u64)rel < limit) atomicAdd(&hist[rel >> shift], 1u);
            };
            for (u32 j = 0; j < L; ++j) {                 // (one list, except for very large tensors)
                const u32 cnt = L == 1u ? S.cand_count : w.cand_ctr[(u64)t * 512u + j * 32u + 1u];
                const u32 i0 = (u32)(((u64)cnt * (a0 - tb)) / tc), i1 = (u32)(((u64)cnt * (a1 - tb)) / tc);
                const EXCP_GLOBAL u32 *c = gptr(w.cand) + w.desc[t].cand_off + (u64)j * cap;
                for (u32 q0 = i0; q0 < i1; q0 += 4u * EXCP_THREADS) {
                    if (q0 + 4u * EXCP_THREADS <= i1) {
                        u32 k[4];
#pragma unroll
                        for (u32 jj = 0; jj < 4; ++jj) k[jj] = c[q0 + jj * EXCP_THREADS + tid];
#pragma unroll
                        for (u32 jj = 0; jj < 4; ++jj) tally(k[jj]);
                    } else {
                        for (u32 i = q0 + tid; i < i1; i += EXCP_THREADS) tally(c[i]);
                    }
                }
            }
            __syncthreads();
            for (u32 i = tid; i < 2048; i += EXCP_THREADS) {
                const u32 v = hist[i];
                if (v) { atomicAdd(&w.med_hist[(u64)t * 2048u + i], v); hist[i] = 0; }
            }
            __syncthreads();
        }
        a0 = a1;
    }
}

__global__ __launch_bounds__(EXCP_THREADS) void k_cand_resolve(Workspace w, GroupParams g) {
    __shared__ u32 s_sum[EXCP_THREADS];
    const u32 t = blockIdx.x, tid = threadIdx.x;
    TState &S = w.st[t];
    if (S.med_state != MED_PENDING || S.sel_width == 0) return;
    u32 *H = w.med_hist + (u64)t * 2048u;
    const u32 width = S.sel_width, shift = width > 11u ? width - 11u : 0u, rank = S.sel_rank, base = S.sel_base;
    if (tid == 0) {
        // the counted bracket values join the listed candidates, each with its multiplicity
        for (u32 q = 0; q < S.natoms; ++q) {
            const u32 rel = S.atom_key[q] - base;
            if ((u64)rel < (1ull << width)) H[rel >> shift] += S.atom_cnt[q];
        }
    }
    __syncthreads();
    u32 c[8], local = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { c[i] = H[tid * 8 + i]; local += c[i]; H[tid * 8 + i] = 0; }
    s_sum[tid] = local;
    __syncthreads();
    for (int off = 1; off < EXCP_THREADS; off <<= 1) {
        u32 v = (tid >= (u32)off) ? s_sum[tid - off] : 0u;
        __syncthreads();
        s_sum[tid] += v;
        __syncthreads();
    }
    const u32 before = s_sum[tid] - local;
    if (rank >= before && rank < before + local) {           // exactly one thread
        u32 r = rank - before;
        int i = 0;
        while (r >= c[i]) { r -= c[i]; ++i; }
        const u32 nb = base + ((u32)(tid * 8 + i) << shift);
        S.sel_base = nb;
        S.sel_width = shift;
        S.sel_rank = r;
        if (shift == 0) { S.med_bits = nb; S.med_state = MED_KNOWN; }
    }
}

// ---------------------------------------------------------------- fallback: select over the whole tensor
template <int PASS>
__global__ __launch_bounds__(EXCP_THREADS) void k_full_hist(Workspace w, GroupParams g) {
    constexpr int NB = (PASS == 2) ? 512 : 2048;
    __shared__ u32 hist[NB];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 G = gridDim.x, b = blockIdx.x;
    const u32 lo = (u32)(((u64)b * g.ntiles) / G), hi = (u32)(((u64)(b + 1) * g.ntiles) / G);
    if (lo >= hi) return;
    for (u32 i = tid; i < NB; i += EXCP_THREADS) hist[i] = 0;
    __syncthreads();
    u32 t = find_owner(w.tile_begin, g.ntensors, lo);
    u32 t_end = w.tile_begin[t + 1];
    bool active = w.st[t].med_state == MED_FALLBACK;
    auto flush = [&](u32 tt) {
        __syncthreads();
        if (active)
            for (u32 i = tid; i < NB; i += EXCP_THREADS) {
                u32 c = hist[i];
                if (c) { atomicAdd(&w.med_hist[(u64)tt * 2048u + i], c); hist[i] = 0; }
            }
        __syncthreads();
    };
    for (u32 tile = lo; tile < hi; ++tile) {
        if (tile >= t_end) {
            flush(t);
            t = find_owner(w.tile_begin, g.ntensors, tile);
            t_end = w.tile_begin[t + 1];
            active = w.st[t].med_state == MED_FALLBACK;
        }
        if (!active) { tile = t_end - 1; continue; }          // skip the rest of this tensor
        const TDesc &D = w.desc[t];
        const u64 n = D.n;
        const u64 base = (u64)(tile - D.tile_begin) * EXCP_TILE;
        const u32 prefix = PASS > 0 ? w.st[t].sel_base : 0u;
        // (this path is taken for heavily tied data above all: see hist_add_tied)
        const u32 rem = (n - base < (u64)EXCP_TILE) ? (u32)(n - base) : EXCP_TILE;
        const u32 wt = excp_wtype(g.flags);
        const bool of_weights = (g.flags & 1u) != 0u;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const u32 off = wave * 1024u + (u32)q * 256u + lane * 4u;
            float a[4], pv[4] = {0.f, 0.f, 0.f, 0.f};
            load_weights4(D.W, base, off, rem, wt, a);
            if (!of_weights) load_weights4(D.Wp, base, off, rem, wt, pv);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool act = off + (u32)j < rem;
                const u32 k = f2u(a[j] - pv[j]) & 0x7fffffffu;
                if (PASS == 0) hist_add_tied(hist, k >> 20, act);
                if (PASS == 1) hist_add_tied(hist, (k >> 9) & 2047u, act && (k >> 20) == prefix);
                if (PASS == 2) hist_add_tied(hist, k & 511u, act && (k >> 9) == prefix);
            }
        }
    }
    flush(t);
}

template <int PASS>
__global__ __launch_bounds__(EXCP_THREADS) void k_full_resolve(Workspace w, GroupParams g) {
    constexpr int NB = (PASS == 2) ? 512 : 2048;
    constexpr int PER = NB / EXCP_THREADS;
    __shared__ u32 s_sum[EXCP_THREADS];
    const u32 t = blockIdx.x, tid = threadIdx.x;
    const u64 n = w.desc[t].n;
    TState &S = w.st[t];
    if (S.med_state != MED_FALLBACK) return;
    u32 *H = w.med_hist + (u64)t * 2048u;
    const u32 rank = (PASS == 0) ? (u32)((n - 1) >> 1) : S.sel_rank;
    const u32 prefix = (PASS == 0) ? 0u : S.sel_base;
    u32 c[PER], local = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) { c[i] = H[tid * PER + i]; local += c[i]; H[tid * PER + i] = 0; }
    s_sum[tid] = local;
    __syncthreads();
    for (int off = 1; off < EXCP_THREADS; off <<= 1) {
        u32 v = (tid >= (u32)off) ? s_sum[tid - off] : 0u;
        __syncthreads();
        s_sum[tid] += v;
        __syncthreads();
    }
    const u32 before = s_sum[tid] - local;
    if (rank >= before && rank < before + local) {           // exactly one thread
        u32 r = rank - before;
        int i = 0;
        while (r >= c[i]) { r -= c[i]; ++i; }
        const u32 bin = tid * PER + i;
        const u32 np = (PASS == 2) ? ((prefix << 9) | bin) : ((prefix << 11) | bin);
        S.sel_base = np;
        S.sel_rank = r;
        if (PASS == 2) { S.med_bits = np; S.med_state = MED_KNOWN; }
    }
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

// The two thresholds of every tensor: t_w = alpha * median, r_o = beta * fp32(exact sum / n).
__global__ void k_thresholds(Workspace w, GroupParams g) {
    const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= g.ntensors) return;
    TState &S = w.st[t];
    const u64 n = w.desc[t].n;
    if (n == 0) { S.med_bits = 0; S.mean32 = 0.f; S.t_w = 0.f; S.r_o = 0.f; S.abs_sum = 0.0; return; }
    const float med = u2f(S.med_bits);
    S.t_w = __fmul_rn(g.alpha, med);
    const double sum = absm_bins_to_double(S.absm);
    const double mean64 = sum / (double)n;
    const float mean32 = (float)mean64;
    S.abs_sum = sum;
    S.mean32 = mean32;
    S.r_o = __fmul_rn(g.beta, mean32);
}

__global__ void k_zero_u32(u32 *p, u64 count) {
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    u64 stride = (u64)gridDim.x * blockDim.x;
    for (; i < count; i += stride) p[i] = 0u;
}

// Plain streaming copy of 16-byte words: a kernel whose HBM traffic is known exactly (bytes read =
// bytes written = the size), used to calibrate the profiler's byte counters.
__global__ __launch_bounds__(256) void k_copy_probe(const uint4 *__restrict__ src, uint4 *__restrict__ dst, u64 count) {
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    const u64 stride = (u64)gridDim.x * blockDim.x;
    for (; i < count; i += stride) dst[i] = src[i];
}

}  // namespace

void launch_copy_probe(const void *src, void *dst, u64 bytes, hipStream_t s) {
    const u64 count = bytes / 16;
    if (!count) return;
    hipLaunchKernelGGL(k_copy_probe, dim3(8192), dim3(256), 0, s, (const uint4 *)src, (uint4 *)dst, count);
}

void launch_zero_u32(u32 *p, u64 count, hipStream_t s) {
    if (!count) return;
    u64 blocks = (count + 1023) / 1024;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_zero_u32, dim3((u32)blocks), dim3(256), 0, s, p, count);
}

// phase 0: sample, 1: streaming pass, 2: bracket check, 3: candidate histogram, 4: candidate resolve,
// 5..7: fallback histograms, 8..10: fallback resolves, 11: thresholds
void launch_stats(const Workspace &w, const GroupParams &g, int phase, hipStream_t s) {
    if (!g.ntensors) return;
    const dim3 block(EXCP_THREADS), per_tensor(g.ntensors), small((g.ntensors + 255) / 256);
    const dim3 stream_grid(excp_grid(w, 8));
    switch (phase) {
        case 0: hipLaunchKernelGGL(k_median_sample, per_tensor, dim3(MED_THREADS), 0, s, w, g); break;
        case 1:
            if (!g.ntiles) break;
            if (g.flags & 0x30u) hipLaunchKernelGGL(k_stats_stream<true>, stream_grid, block, 0, s, w, g);
            else hipLaunchKernelGGL(k_stats_stream<false>, stream_grid, block, 0, s, w, g);
            break;
        case 2: hipLaunchKernelGGL(k_cand_begin, small, dim3(256), 0, s, w, g); break;
        case 3: if (g.ntiles) hipLaunchKernelGGL(k_cand_hist, dim3((g.ntiles + CAND_TILES - 1) / CAND_TILES), block, 0, s, w, g); break;
        case 4: hipLaunchKernelGGL(k_cand_resolve, per_tensor, block, 0, s, w, g); break;
        case 5: if (g.ntiles) hipLaunchKernelGGL(k_full_hist<0>, stream_grid, block, 0, s, w, g); break;
        case 6: if (g.ntiles) hipLaunchKernelGGL(k_full_hist<1>, stream_grid, block, 0, s, w, g); break;
        case 7: if (g.ntiles) hipLaunchKernelGGL(k_full_hist<2>, stream_grid, block, 0, s, w, g); break;
        case 8: hipLaunchKernelGGL(k_full_resolve<0>, per_tensor, block, 0, s, w, g); break;
        case 9: hipLaunchKernelGGL(k_full_resolve<1>, per_tensor, block, 0, s, w, g); break;
        case 10: hipLaunchKernelGGL(k_full_resolve<2>, per_tensor, block, 0, s, w, g); break;
        case 11: hipLaunchKernelGGL(k_thresholds, small, dim3(256), 0, s, w, g); break;
        default: break;
    }
}
