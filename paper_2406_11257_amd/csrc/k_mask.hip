// Joint pruning masks (Sec. 3.2, Eq. "r_w" and Eq. "r_o") and the order-preserving compaction of
// the survivors.
//
// Pass A (k_mask_slots) reads W_prev, W_t, m and v once.  Work unit: a sub-tile of 2048 elements
// (half a 4096-element tile), owned by one wave, which writes the keep bitmap, the sub-tile's
// survivor counts, and the survivors themselves -- in index order, together with their M_o bits --
// into the sub-tile's own slot of a scratch area.  No wave waits for another: where a survivor
// finally goes depends on the counts of all earlier sub-tiles, and that is left to a scan
// (k_mask_scan over the sub-tile counts of every tensor) and to pass B (k_mask_gather), which copies
// every slot to its place in the dense survivor arrays; k_mask_bitmap_o then assembles bitmap_o from
// the sub-tiles' local bit streams.  The extra copy costs 8 bytes per survivor; it replaces a chained
// scan whose waits cost more than that.
#include "excp_util.h"

namespace {

constexpr u32 SUB = 2048;          // elements per sub-tile
constexpr u32 QUARTER = 512;       // elements a wave holds at once: 8 batches of 64
constexpr int NBATCH = 8;          // 64-element batches per quarter
constexpr u32 BO_WORDS = SUB / 64; // M_o words kept per sub-tile

// The bits of one quarter as they arrive (weights as stored: fp32 bit patterns, or 16-bit values).
struct Regs {
    u32 w[NBATCH], p[NBATCH];
    float m[NBATCH], v[NBATCH];
};

// What a wave needs to know about the sub-tile it works on (all of it the same in every lane).
struct SubTile {
    u64 n, base;                   // elements of the tensor; first element of the sub-tile inside it
    float t_w, r_o;                // the tensor's thresholds
    float T_keep, T_drop;          // t_w^2 with the estimate's guard band on either side
    bool T_ok;                     // t_w^2 is a positive normal number: the estimate may be used at all
    EXCP_GLOBAL float *sw, *sm, *sv;   // the sub-tile's slot in the three survivor areas
    u64 *bm;                       // the tensor's keep bitmap (inside its blob)
    u64 *bo;                       // the sub-tile's 32 local M_o words
};

// Loads of one quarter (512 elements starting at element `first` of the tensor) that lies wholly
// inside the tensor: one base per array, the batches are immediate offsets.
template <bool W16>
__device__ __forceinline__ void load_quarter(Regs &R, const TDesc &D, u64 first, u32 lane) {
    const EXCP_GLOBAL float *gM = gptr(D.m) + first, *gV = gptr(D.v) + first;
    if (W16) {
        const EXCP_GLOBAL unsigned short *hW = gptr((const unsigned short *)D.W) + first;
        const EXCP_GLOBAL unsigned short *hP = gptr((const unsigned short *)D.Wp) + first;
#pragma unroll
        for (int j = 0; j < NBATCH; ++j) { R.w[j] = hW[j * 64 + lane]; R.p[j] = hP[j * 64 + lane]; }
    } else {
        const EXCP_GLOBAL u32 *gW = gptr((const u32 *)D.W) + first, *gP = gptr((const u32 *)D.Wp) + first;
#pragma unroll
        for (int j = 0; j < NBATCH; ++j) { R.w[j] = gW[j * 64 + lane]; R.p[j] = gP[j * 64 + lane]; }
    }
#pragma unroll
    for (int j = 0; j < NBATCH; ++j) { R.m[j] = gM[j * 64 + lane]; R.v[j] = gV[j * 64 + lane]; }
}

// The same for a quarter of which only `rem` elements exist (a tensor's ragged end; rem may be 0).
template <bool W16>
__device__ __forceinline__ void load_quarter_ragged(Regs &R, const TDesc &D, u64 first, u32 rem, u32 lane) {
#pragma unroll
    for (int j = 0; j < NBATCH; ++j) {
        const u32 e = (u32)j * 64u + lane;
        const bool ok = e < rem;
        const u64 idx = first + e;
        R.w[j] = ok ? (W16 ? (u32)((const unsigned short *)D.W)[idx] : ((const u32 *)D.W)[idx]) : 0u;
        R.p[j] = ok ? (W16 ? (u32)((const unsigned short *)D.Wp)[idx] : ((const u32 *)D.Wp)[idx]) : 0u;
        R.m[j] = ok ? D.m[idx] : 0.f;
        R.v[j] = ok ? D.v[idx] : 1.f;
    }
}

// Quarter r (0..3) of a sub-tile: decisions, bitmap words, survivors to their ranks.  All lanes of the
// wave are active throughout: every decision is first a wave-wide bit mask (the ballot of one
// comparison), the masks are combined as 64-bit integers, and only the final masks become lane
// predicates again.  rem = elements of the quarter that exist (FULL: all 512).
// cw_run / co_run / nf_run: kept residuals, kept moments and non-finite v of the sub-tile so far.
template <bool NW2M, bool W16, bool FULL>
__device__ __forceinline__ void mask_quarter(const Regs &R, const SubTile &S, u32 r, u32 rem, u32 flags, u32 *my_bo,
                                             u32 lane, u32 &cw_run, u32 &co_run, u32 &nf_run) {
    const bool bf = W16 && excp_wtype(flags) == 2u;
    u32 w_lo = 0, w_hi = 0, o_lo = 0, o_hi = 0;          // lane j: the j-th bitmap word of this quarter
#pragma unroll
    for (int j = 0; j < NBATCH; ++j) {
        // lanes whose element exists (all of them, except at a tensor's ragged end)
        const u32 left = FULL ? 64u : (rem > (u32)j * 64u ? rem - (u32)j * 64u : 0u);
        const u64 valid = left >= 64u ? ~0ull : ((1ull << left) - 1ull);
        const float wv = W16 ? w16_widen(R.w[j], bf) : u2f(R.w[j]);
        const float pv = W16 ? w16_widen(R.p[j], bf) : u2f(R.p[j]);
        const float d = wv - pv;                          // the residual
        const float ad = fabsf(d), vv = R.v[j], mv = R.m[j];
        u64 bw;
        if (flags & 2u) {
            bw = ballot64(ad > S.t_w);                    // ablation: the same scalar threshold for every element
        } else {
            // (d^2 may underflow where d^2 v does not: every factor and product must be a positive normal number)
            const float dd = ad * ad, x = dd * vv;
            const u64 b_keep = ballot64(x > S.T_keep), b_drop = ballot64(x < S.T_drop);
            const u64 b_trust = ballot64(__builtin_amdgcn_classf(vv, 0x100)) & ballot64(__builtin_amdgcn_classf(dd, 0x100)) &
                                ballot64(__builtin_amdgcn_classf(x, 0x100));
            const u64 amb = S.T_ok ? (~(b_keep | b_drop) | ~b_trust) : ~0ull;
            bw = b_keep;
            if (amb & valid) {
                // sqrtf and '/' are the correctly rounded forms (the build passes
                // -fhip-fp32-correctly-rounded-divide-sqrt); __fsqrt_rn is NOT on this target
                const u64 b_exact = ballot64(ad > S.t_w / sqrtf(vv));
                bw = (b_keep & ~amb) | (b_exact & amb);
            }
        }
        bw &= valid;
        nf_run += (u32)__popcll(ballot64((f2u(vv) & 0x7f800000u) == 0x7f800000u) & valid);
        const u64 bo = ballot64(fabsf(mv) > S.r_o) & (NW2M ? valid : bw);
        if (lane == (u32)j) { w_lo = (u32)bw; w_hi = (u32)(bw >> 32); }
        const u32 rk = cw_run + __builtin_amdgcn_mbcnt_hi((u32)(bw >> 32), __builtin_amdgcn_mbcnt_lo((u32)bw, 0u));
        if (__builtin_amdgcn_inverse_ballot_w64(bw)) S.sw[rk] = d;
        if (__builtin_amdgcn_inverse_ballot_w64(bo)) {
            const u32 ro = co_run + __builtin_amdgcn_mbcnt_hi((u32)(bo >> 32), __builtin_amdgcn_mbcnt_lo((u32)bo, 0u));
            S.sm[ro] = mv; S.sv[ro] = vv;
            if (!NW2M) atomicOr(&my_bo[rk >> 5], 1u << (rk & 31u));
        }
        if (NW2M && lane == (u32)j) { o_lo = (u32)bo; o_hi = (u32)(bo >> 32); }
        cw_run += (u32)__popcll(bw);
        co_run += (u32)__popcll(bo);
    }
    // the quarter's eight words of the keep bitmap; words past the last element carry an all-zero
    // ballot: that is the section's 16-byte padding
    const u64 nwords = excp_words(S.n), word = ((S.base + (u64)r * QUARTER) >> 6) + lane;
    if (lane < (u32)NBATCH && (FULL || word < nwords + (nwords & 1ull))) S.bm[word] = (u64)w_lo | ((u64)w_hi << 32);
    if (NW2M && lane < (u32)NBATCH) S.bo[r * NBATCH + lane] = (u64)o_lo | ((u64)o_hi << 32);
}

// Pass A.  A wave owns whole sub-tiles (a contiguous range of the group's sub-tile list) and walks each
// in four quarters of 512 elements; lane l of batch j holds element 64 j + l, so a wave ballot is one
// word of a bitmap.  Nothing is shared between waves: no barrier after the tile table is loaded.
// While one quarter is worked on the next is already on its way from memory (two register sets).
//
// Per element: the residual; the keep decision |d| > t_w / sqrt(v) with correctly rounded sqrt and
// divide -- taken from the estimate d^2 v against t_w^2 when that is not within 1e-5 of the boundary
// (the estimate's own error is below 3e-7) and from the exact expression otherwise, so it is always
// that of the exact expression; the M_o decision.  Survivors go straight to their rank in the
// sub-tile's slot (ballot + lane count); the M_o bit of a kept residual is ORed into the wave's own
// LDS words at the residual's rank.
//
// NW2M (Table "vit", no weights-to-momentum check): M_o(i) = |m_i| > r_o for every element, kept
// weight or not; the sub-tile's M_o words are then indexed by element and are the ballots themselves.
// W16: the two weight arrays hold 16-bit values (fp16 or bf16 by the flags), widened as they are used.
template <bool NW2M, bool W16>
__global__ __launch_bounds__(EXCP_THREADS, 5) void k_mask_slots(Workspace w, GroupParams g) {
    __shared__ u32 s_bo[EXCP_THREADS / 64][SUB / 32];      // per wave: M_o bits of its sub-tile's kept residuals, by rank
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    const u32 lane = threadIdx.x & 63u;
    const u32 wave = (u32)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const u32 nsub = 2u * g.ntiles;
    load_tile_table(s_tiles, w.tile_begin, g.ntensors);
    const u32 nwaves = gridDim.x * (EXCP_THREADS / 64), wid = blockIdx.x * (EXCP_THREADS / 64) + wave;
    const u32 sub_lo = (u32)(((u64)wid * nsub) / nwaves), sub_hi = (u32)(((u64)(wid + 1u) * nsub) / nwaves);
    if (sub_lo >= sub_hi) return;
    u32 *my_bo = s_bo[wave];
    my_bo[lane] = 0u;
    u32 t = 0, first_sub = 0, end_sub = 0;                // the tensor in hand, its first sub-tile, one past its last
    Regs A, B;
    for (u32 sub = sub_lo; sub < sub_hi; ++sub) {
        if (sub >= end_sub) {                             // (looked up again only when a tensor's sub-tiles run out)
            t = (u32)__builtin_amdgcn_readfirstlane((int)find_owner(s_tiles, g.ntensors, sub >> 1));
            first_sub = (u32)__builtin_amdgcn_readfirstlane((int)(2u * s_tiles[t]));
            end_sub = (u32)__builtin_amdgcn_readfirstlane((int)(2u * s_tiles[t + 1u]));
        }
        // The tensor's description and thresholds are not written by this kernel: read as constant
        // memory they come through the scalar unit, which global memory that the kernel also
        // stores to may not.
        const EXCP_CONSTANT TDesc *Dc = (const EXCP_CONSTANT TDesc *)(uintptr_t)(w.desc + t);
        const EXCP_CONSTANT TState *St = (const EXCP_CONSTANT TState *)(uintptr_t)(w.st + t);
        TDesc D;
        D.Wp = Dc->Wp; D.W = Dc->W; D.m = Dc->m; D.v = Dc->v; D.n = Dc->n; D.blob = Dc->blob; D.elem_off = Dc->elem_off;
        SubTile S;
        S.n = D.n; S.base = (u64)(sub - first_sub) * SUB;
        S.t_w = St->t_w; S.r_o = St->r_o;
        const float T = S.t_w * S.t_w;
        S.T_keep = T * 1.00001f; S.T_drop = T * 0.99999f; S.T_ok = __builtin_amdgcn_classf(T, 0x100);
        const u64 slot = D.elem_off + S.base;
        S.sw = gptr(w.pw) + slot; S.sm = gptr(w.pm) + slot; S.sv = gptr(w.pv) + slot;
        S.bm = (u64 *)(D.blob + EXCP_HEADER + excp_books_bytes((u32)g.nbits));
        S.bo = w.mask_bo + (u64)sub * BO_WORDS;
        u32 cw_run = 0, co_run = 0, nf_run = 0;
        if (S.base + SUB <= S.n) {
            load_quarter<W16>(A, D, S.base, lane);
            load_quarter<W16>(B, D, S.base + QUARTER, lane);
            mask_quarter<NW2M, W16, true>(A, S, 0u, QUARTER, g.flags, my_bo, lane, cw_run, co_run, nf_run);
            load_quarter<W16>(A, D, S.base + 2u * QUARTER, lane);
            mask_quarter<NW2M, W16, true>(B, S, 1u, QUARTER, g.flags, my_bo, lane, cw_run, co_run, nf_run);
            load_quarter<W16>(B, D, S.base + 3u * QUARTER, lane);
            mask_quarter<NW2M, W16, true>(A, S, 2u, QUARTER, g.flags, my_bo, lane, cw_run, co_run, nf_run);
            mask_quarter<NW2M, W16, true>(B, S, 3u, QUARTER, g.flags, my_bo, lane, cw_run, co_run, nf_run);
        } else {
#pragma unroll 1
            for (u32 r = 0; r < 4u; ++r) {
                const u64 first = S.base + (u64)r * QUARTER;
                const u32 rem = S.n > first ? (S.n - first < (u64)QUARTER ? (u32)(S.n - first) : QUARTER) : 0u;
                load_quarter_ragged<W16>(A, D, first, rem, lane);
                mask_quarter<NW2M, W16, false>(A, S, r, rem, g.flags, my_bo, lane, cw_run, co_run, nf_run);
            }
        }
        // the sub-tile is complete: its M_o words (by survivor rank) and its counts
        if (!NW2M) {
            const u64 word = (u64)my_bo[2u * (lane & 31u)] | ((u64)my_bo[2u * (lane & 31u) + 1u] << 32);
            if (lane < ((cw_run + 63u) >> 6)) S.bo[lane] = word;
            my_bo[lane] = 0u;
        }
        if (lane == 0u) {
            w.tile_status[sub] = ((u64)cw_run << 32) | (u64)co_run;
            if (nf_run) atomicAdd(&w.st[t].nonfinite, (u64)nf_run);
        }
    }
}

// One wave copies floats in batches of N x 64; every load of a batch is issued before its stores so
// that a copy is not a chain of dependent round trips.
template <int N>
__device__ __forceinline__ void load_batch(float (&q)[N], const EXCP_GLOBAL float *src, u32 cnt, u32 b0, u32 lane) {
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const u32 i = b0 + (u32)k * 64u + lane;
        q[k] = i < cnt ? src[i] : 0.f;
    }
}
template <int N>
__device__ __forceinline__ void store_batch(EXCP_GLOBAL float *dst, const float (&q)[N], u32 cnt, u32 b0, u32 lane) {
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const u32 i = b0 + (u32)k * 64u + lane;
        if (i < cnt) dst[i] = q[k];
    }
}

// Exclusive scan of the sub-tile counts of every tensor; the totals are the tensor's n_w and n_o.
// Counts are packed (survivors << 32 | moment survivors).  A tensor's sub-tiles are cut into sixteen
// parts, one workgroup each: first the parts' totals, then every workgroup scans its own part from the
// sum of the parts before it.
constexpr u32 MSCAN_PARTS = 16;

__device__ __forceinline__ void mscan_range(u32 nsub, u32 part, u32 &s0, u32 &s1) {
    const u32 per = ((nsub + MSCAN_PARTS - 1u) / MSCAN_PARTS + 3u) & ~3u;
    s0 = min(part * per, nsub);
    s1 = min(s0 + per, nsub);
}

__global__ __launch_bounds__(EXCP_THREADS) void k_mask_scan_parts(Workspace w, GroupParams g) {
    __shared__ u64 s_sum[EXCP_THREADS / 64];
    const u32 t = blockIdx.x / MSCAN_PARTS, part = blockIdx.x % MSCAN_PARTS, tid = threadIdx.x;
    const TDesc &D = w.desc[t];
    u32 s0, s1;
    mscan_range(2u * D.tile_count, part, s0, s1);
    const u64 *cnt = w.tile_status + 2ull * D.tile_begin;
    u64 local = 0;
    for (u32 i = s0 + tid; i < s1; i += EXCP_THREADS) local += cnt[i];
    local = wave_sum_u64(local);
    if ((tid & 63u) == 0u) s_sum[tid >> 6] = local;
    __syncthreads();
    if (tid == 0) w.mask_part[(u64)t * MSCAN_PARTS + part] = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
}

__global__ __launch_bounds__(EXCP_THREADS) void k_mask_scan(Workspace w, GroupParams g) {
    __shared__ u64 s_sum[EXCP_THREADS];
    const u32 t = blockIdx.x / MSCAN_PARTS, part = blockIdx.x % MSCAN_PARTS, tid = threadIdx.x;
    const TDesc &D = w.desc[t];
    const u32 nsub = 2u * D.tile_count;
    u32 s0, s1;
    mscan_range(nsub, part, s0, s1);
    u64 *cnt = w.tile_status + 2ull * D.tile_begin;
    u64 carry = 0;
    for (u32 q = 0; q < part; ++q) carry += w.mask_part[(u64)t * MSCAN_PARTS + q];
    if (part == MSCAN_PARTS - 1u && tid == 0) {
        const u64 total = carry + w.mask_part[(u64)t * MSCAN_PARTS + part];
        w.st[t].n_w = total >> 32; w.st[t].n_o = total & 0xffffffffull;
    }
    for (u32 base = s0; base < s1; base += EXCP_THREADS * 4) {
        // four consecutive sub-tiles per thread
        u64 v[4], local = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32 i = base + tid * 4 + q;
            v[q] = (i < s1) ? cnt[i] : 0ull;
            local += v[q];
        }
        s_sum[tid] = local;
        __syncthreads();
        for (int off = 1; off < EXCP_THREADS; off <<= 1) {
            u64 a = (tid >= (u32)off) ? s_sum[tid - off] : 0ull;
            __syncthreads();
            s_sum[tid] += a;
            __syncthreads();
        }
        u64 run = carry + s_sum[tid] - local;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32 i = base + tid * 4 + q;
            if (i < s1) w.mask_prefix[2ull * D.tile_begin + i] = run;
            run += v[q];
        }
        carry += s_sum[EXCP_THREADS - 1];
        __syncthreads();
    }
}

// Pass B: one wave per sub-tile copies the slot to its place in the dense survivor arrays.  A workgroup takes a
// contiguous range of batches of 32 consecutive sub-tiles; a batch's counts, prefixes and tensor data are
// fetched once, side by side, into LDS, so that a wave's copies do not wait behind a chain of dependent
// look-ups.
// The same pass counts, for the value partition of the codebook stage, how many of the values it moves
// fall into each of the 256 value buckets (the map k_km_sample made from the slots): the values are in
// registers here, and a pass of its own would read them all again.  Counts are kept per 16 chunks
// (131 072 positions) of a stream, in the row of the first of those chunks; the scatter's workgroups
// begin only at such positions.  A workgroup adds up in LDS as long as its batches stay inside one tensor
// and one such unit per stream, and hands the sums over when that changes.
constexpr u32 GATHER_SUBS = 32;
constexpr u32 SUPER_SHIFT = 17;                          // log2 of the positions per counted unit
static_assert((1u << SUPER_SHIFT) == EXCP_SUPER_CHUNKS * EXCP_CHUNK, "counted unit = EXCP_SUPER_CHUNKS chunks");

__global__ __launch_bounds__(EXCP_THREADS) void k_mask_gather(Workspace w, GroupParams g) {
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    __shared__ u32 s_tw[GATHER_SUBS], s_to[GATHER_SUBS], s_pw[GATHER_SUBS], s_po[GATHER_SUBS], s_t[GATHER_SUBS];
    __shared__ u64 s_slot[GATHER_SUBS], s_eoff[GATHER_SUBS];
    __shared__ u32 s_map[3][EXCP_KM_MAP_WORDS];
    __shared__ u32 s_hist[3][2][256];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 nsub = 2u * g.ntiles;
    const bool counting = (g.flags & 4u) == 0u;          // (no codebooks without quantisation)
    load_tile_table(s_tiles, w.tile_begin, g.ntensors);
    const u32 nbatch = (nsub + GATHER_SUBS - 1u) / GATHER_SUBS;
    const u32 b_lo = (u32)(((u64)blockIdx.x * nbatch) / gridDim.x), b_hi = (u32)(((u64)(blockIdx.x + 1u) * nbatch) / gridDim.x);
    for (u32 i = tid; i < 3u * 2u * 256u; i += EXCP_THREADS) (&s_hist[0][0][0])[i] = 0;
    u32 cur_t = 0xffffffffu, cur_sc[3] = {0u, 0u, 0u};   // what the LDS counts belong to
    bool live[3] = {false, false, false};                // the stream has a place in the chunk list (its tensor did not fail)
    // hands the counts over: thread b adds bucket b of both units of the three streams
    auto flush = [&]() {
        __syncthreads();
        if (cur_t != 0xffffffffu) {
#pragma unroll
            for (u32 k = 0; k < 3; ++k) {
                if (!live[k]) continue;
                const u32 row0 = w.seg[3u * cur_t + k].chunk_begin + cur_sc[k] * EXCP_SUPER_CHUNKS;
#pragma unroll
                for (u32 u = 0; u < 2; ++u) {
                    const u32 h = s_hist[k][u][tid];
                    if (h) { atomicAdd(&w.km_cnt[(u64)(row0 + u * EXCP_SUPER_CHUNKS) * 256u + tid], h); s_hist[k][u][tid] = 0; }
                }
            }
        }
        __syncthreads();
    };
    for (u32 batch = b_lo; batch < b_hi; ++batch) {
        const u32 sub0 = batch * GATHER_SUBS;
        __syncthreads();
        if (tid < GATHER_SUBS) {
            const u32 sub = sub0 + tid;
            u32 tw = 0, to = 0;
            if (sub < nsub) {
                const u64 c = w.tile_status[sub], pre = w.mask_prefix[sub];
                tw = (u32)(c >> 32); to = (u32)c;
                const u32 t = find_owner(s_tiles, g.ntensors, sub >> 1);
                const u64 eoff = w.desc[t].elem_off;
                s_pw[tid] = (u32)(pre >> 32); s_po[tid] = (u32)pre; s_t[tid] = t;
                s_eoff[tid] = eoff;
                s_slot[tid] = eoff + (u64)(sub - 2u * s_tiles[t]) * SUB;
            }
            s_tw[tid] = tw; s_to[tid] = to;
        }
        __syncthreads();
        const u32 nvalid = min(GATHER_SUBS, nsub - sub0);
        const u32 t0 = s_t[0];
        const bool one_tensor = t0 == s_t[nvalid - 1u];
        if (counting) {
            if (one_tensor) {
                const u32 sc[3] = {s_pw[0] >> SUPER_SHIFT, s_po[0] >> SUPER_SHIFT, s_po[0] >> SUPER_SHIFT};
                if (t0 != cur_t || sc[0] != cur_sc[0] || sc[1] != cur_sc[1]) {
                    flush();
                    if (t0 != cur_t) {
#pragma unroll
                        for (u32 k = 0; k < 3; ++k) {
                            live[k] = w.seg[3u * t0 + k].len != 0;
                            if (live[k])
                                for (u32 i = tid; i < EXCP_KM_MAP_WORDS; i += EXCP_THREADS) s_map[k][i] = w.km_split[(u64)(3u * t0 + k) * EXCP_KM_MAP_WORDS + i];
                        }
                    }
                    cur_t = t0; cur_sc[0] = sc[0]; cur_sc[1] = sc[1]; cur_sc[2] = sc[2];
                    __syncthreads();
                }
            } else if (cur_t != 0xffffffffu) {
                flush();
                cur_t = 0xffffffffu;
            }
        }
        const bool in_lds = counting && one_tensor;
        u32 par[3][4] = {};                              // the maps' four parameters, out of LDS once per batch
        if (in_lds) {
#pragma unroll
            for (u32 k = 0; k < 3; ++k)
                if (live[k]) { par[k][0] = s_map[k][0]; par[k][1] = s_map[k][1]; par[k][2] = s_map[k][2]; par[k][3] = s_map[k][3]; }
        }
        for (u32 j = wave; j < nvalid; j += 4) {
            const u32 tw = s_tw[j], to = s_to[j];
            if (tw == 0 && to == 0) continue;
            const u32 pw = s_pw[j], po = s_po[j];
            const u64 slot = s_slot[j], eoff = s_eoff[j];
            const EXCP_GLOBAL float *sw = gptr(w.pw) + slot, *sm = gptr(w.pm) + slot, *sv = gptr(w.pv) + slot;
            EXCP_GLOBAL float *xw = gptr(w.xw) + eoff + pw;
            EXCP_GLOBAL float *xm = gptr(w.xm) + eoff + po;
            EXCP_GLOBAL float *xv = gptr(w.xv) + eoff + po;
            // counts of a batch that holds the end of one tensor and the start of the next (small tensors) go
            // straight to the table, with that tensor's maps read where they are: what a stream needs for
            // that is fetched once per sub-tile
            const u32 tj = s_t[j];
            u32 g_row[3] = {0u, 0u, 0u}, g_par[3][4] = {};
            bool g_live[3] = {false, false, false};
            const EXCP_GLOBAL unsigned char *g_cells[3] = {nullptr, nullptr, nullptr};
            if (counting && !in_lds) {
#pragma unroll
                for (u32 k = 0; k < 3; ++k) {
                    const u32 sg = 3u * tj + k;
                    g_live[k] = w.seg[sg].len != 0;
                    g_row[k] = w.seg[sg].chunk_begin;
                    const u32 *mp = w.km_split + (u64)sg * EXCP_KM_MAP_WORDS;
                    if (g_live[k]) { g_par[k][0] = mp[0]; g_par[k][1] = mp[1]; g_par[k][2] = mp[2]; g_par[k][3] = mp[3]; }
                    g_cells[k] = gptr((const unsigned char *)(mp + 4));
                }
            }
            auto count = [&](u32 k, float x, u32 place) {
                if (in_lds) {
                    if (live[k]) atomicAdd(&s_hist[k][(place >> SUPER_SHIFT) != cur_sc[k] ? 1u : 0u][((const unsigned char *)(s_map[k] + 4))[cell_of(x, par[k])]], 1u);
                } else if (g_live[k]) {
                    const u32 row = g_row[k] + (place >> SUPER_SHIFT) * EXCP_SUPER_CHUNKS;
                    atomicAdd(&w.km_cnt[(u64)row * 256u + g_cells[k][cell_of(x, g_par[k])]], 1u);
                }
            };
            {
                // the first batch of all three runs in flight together (usually there is no second)
                float qw[12], qm[4], qv[4];
                load_batch<12>(qw, sw, tw, 0, lane); load_batch<4>(qm, sm, to, 0, lane); load_batch<4>(qv, sv, to, 0, lane);
                store_batch<12>(xw, qw, tw, 0, lane); store_batch<4>(xm, qm, to, 0, lane); store_batch<4>(xv, qv, to, 0, lane);
                if (counting) {
#pragma unroll
                    for (u32 k = 0; k < 12; ++k) { const u32 i = k * 64u + lane; if (i < tw) count(0, qw[k], pw + i); }
#pragma unroll
                    for (u32 k = 0; k < 4; ++k) { const u32 i = k * 64u + lane; if (i < to) { count(1, qm[k], po + i); count(2, qv[k], po + i); } }
                }
                for (u32 b0 = 768u; b0 < tw; b0 += 768u) {
                    load_batch<12>(qw, sw, tw, b0, lane); store_batch<12>(xw, qw, tw, b0, lane);
                    if (counting) {
#pragma unroll
                        for (u32 k = 0; k < 12; ++k) { const u32 i = b0 + k * 64u + lane; if (i < tw) count(0, qw[k], pw + i); }
                    }
                }
                for (u32 b0 = 256u; b0 < to; b0 += 256u) {
                    load_batch<4>(qm, sm, to, b0, lane); load_batch<4>(qv, sv, to, b0, lane);
                    store_batch<4>(xm, qm, to, b0, lane); store_batch<4>(xv, qv, to, b0, lane);
                    if (counting) {
#pragma unroll
                        for (u32 k = 0; k < 4; ++k) { const u32 i = b0 + k * 64u + lane; if (i < to) { count(1, qm[k], po + i); count(2, qv[k], po + i); } }
                    }
                }
            }
        }
    }
    if (counting) flush();
}

// bitmap_o (the M_o bits of the survivors, in survivor order) from the sub-tiles' local bit
// streams.  Output-centric: one lane builds one 64-bit word from the one to three sub-tiles whose
// survivors it covers, so the words are written whole, once, with no atomics; a wave takes 64
// consecutive words (4096 survivor positions) of one tensor.  The sub-tile that holds the wave's
// first position is found by a 64-way search over the tensor's scanned survivor counts.
__global__ __launch_bounds__(EXCP_THREADS) void k_mask_bitmap_o(Workspace w, GroupParams g) {
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    __shared__ u32 s_P[4][65], s_c[4][64];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    load_tile_table(s_tiles, w.tile_begin, g.ntensors);
    for (u32 blk = blockIdx.x * 4 + wave; blk < g.ntiles; blk += gridDim.x * 4) {
        const u32 t = find_owner(s_tiles, g.ntensors, blk);
        const u32 b = blk - s_tiles[t];                     // the tensor's b-th run of 64 words
        const u32 n_w = (u32)w.st[t].n_w;
        const u32 nwo = (u32)excp_words(n_w), padded = nwo + (nwo & 1u);   // section length, zero-padded to 16 bytes
        if (64u * b >= padded) continue;
        const TDesc &D = w.desc[t];
        const u64 off_bo = EXCP_HEADER + excp_books_bytes((u32)g.nbits) + excp_pad16(8ull * excp_words(D.n));
        const u64 cap_words = (D.blob_cap > off_bo) ? (D.blob_cap - off_bo) >> 3 : 0ull;
        const u32 sb = 2u * s_tiles[t], se = 2u * s_tiles[t + 1];
        const u32 Q0 = 4096u * b;
        // last sub-tile whose first survivor position is <= Q0 (positions are non-decreasing)
        u32 lo = sb, hi = se;
        while (hi - lo > 1u) {
            const u32 span = hi - lo - 1u;                  // open choices lo + 1 .. hi - 1
            const bool act = span > 64u || lane < span;
            const u32 idx = span > 64u ? lo + 1u + (u32)(((u64)span * lane) >> 6) : lo + 1u + lane;
            const u32 P = act ? (u32)(w.mask_prefix[idx] >> 32) : 0xffffffffu;
            const u64 le = ballot64(act && P <= Q0);        // a run of ones from lane 0 up
            const u32 cnt = __popcll(le), nact = span > 64u ? 64u : span;
            const u32 up = __shfl(idx, cnt ? cnt - 1u : 0u, WAVE), dn = __shfl(idx, cnt < 64u ? cnt : 63u, WAVE);
            if (cnt < nact) hi = dn;
            if (cnt) lo = up;
        }
        const u32 s0 = lo;
        // the next 64 sub-tiles: first survivor position and survivor count, side by side in LDS
        {
            const u32 si = s0 + lane;
            const bool in = si < se;
            s_P[wave][lane] = in ? (u32)(w.mask_prefix[si] >> 32) : 0xffffffffu;
            s_c[wave][lane] = in ? (u32)(w.tile_status[si] >> 32) : 0u;
            if (lane == 0) s_P[wave][64] = 0xffffffffu;
        }
        const u32 widx = 64u * b + lane;
        if (widx >= padded) continue;
        u64 word = 0;
        if (widx < nwo) {
            const u32 Q = widx * 64u;                        // this word covers survivor positions [Q, Q + 64)
            u32 i = 0;                                       // last entry of the window with position <= Q
#pragma unroll
            for (u32 step = 32; step >= 1; step >>= 1) if (s_P[wave][i + step] <= Q) i += step;
            for (;; ++i) {
                const u32 cur = s0 + i;
                if (cur >= se) break;
                const u32 P = i < 64u ? s_P[wave][i] : (u32)(w.mask_prefix[cur] >> 32);
                if (P >= Q + 64u) break;
                const u32 c = i < 64u ? s_c[wave][i] : (u32)(w.tile_status[cur] >> 32);
                if (P + c <= Q) continue;                    // ends before this word (or is empty)
                const u32 a = max(Q, P), e = min(Q + 64u, P + c);      // overlap, in survivor positions
                const u32 la = a - P, len = e - a;           // first local bit, number of bits
                const u64 *loc = w.mask_bo + (u64)cur * BO_WORDS;
                const u32 k = la >> 6, sh = la & 63u;
                const u64 w0 = loc[k];
                const u64 w1 = ((k + 1u) * 64u < c) ? loc[k + 1u] : 0ull;
                u64 bits = sh ? ((w0 >> sh) | (w1 << (64u - sh))) : w0;
                if (len < 64u) bits &= (1ull << len) - 1ull;
                word |= bits << (a - Q);
            }
        }
        if (widx < cap_words) ((u64 *)(D.blob + off_bo))[widx] = word;
    }
}

// bitmap_o without the weights-to-momentum check: one bit per element, so the sub-tiles' words are
// already the section's words, 32 per sub-tile.
__global__ __launch_bounds__(EXCP_THREADS) void k_mask_bitmap_o_elems(Workspace w, GroupParams g) {
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    load_tile_table(s_tiles, w.tile_begin, g.ntensors);
    for (u32 blk = blockIdx.x * 4 + wave; blk < g.ntiles; blk += gridDim.x * 4) {
        const u32 t = find_owner(s_tiles, g.ntensors, blk);
        const u32 b = blk - s_tiles[t];                     // the tensor's b-th tile = 64 words
        const TDesc &D = w.desc[t];
        const u64 nwo = excp_words(D.n), padded = nwo + (nwo & 1ull);
        const u64 widx = 64ull * b + lane;
        if (widx >= padded) continue;
        const u64 off_bo = EXCP_HEADER + excp_books_bytes((u32)g.nbits) + excp_pad16(8ull * nwo);
        const u64 cap_words = (D.blob_cap > off_bo) ? (D.blob_cap - off_bo) >> 3 : 0ull;
        const u64 word = widx < nwo ? w.mask_bo[(2ull * blk + (lane >> 5)) * BO_WORDS + (lane & 31u)] : 0ull;
        if (widx < cap_words) ((u64 *)(D.blob + off_bo))[widx] = word;
    }
}

// After the masks: blob section offsets, capacity check, survivor stream lengths and the chunk
// list of the survivor passes.  One workgroup; tensors and streams are few.
__global__ __launch_bounds__(EXCP_THREADS) void k_layout(Workspace w, GroupParams g, u32 *seg_chunk_begin) {
    __shared__ u32 s_sum[EXCP_THREADS];
    const u32 tid = threadIdx.x;
    const u32 nseg = 3u * g.ntensors;
    const u32 per = (nseg + EXCP_THREADS - 1) / EXCP_THREADS;
    u32 local = 0;
    for (u32 q = 0; q < per; ++q) {
        u32 sidx = tid * per + q;
        if (sidx >= nseg) break;
        u32 t = sidx / 3u, which = sidx % 3u;
        TState &S = w.st[t];
        const TDesc &D = w.desc[t];
        if (which == 0) {
            const u64 n = D.n, nw = S.n_w, no = S.n_o, nb = (u64)g.nbits;
            u64 off = EXCP_HEADER + excp_books_bytes((u32)g.nbits) + excp_pad16(8ull * excp_words(n));
            S.off_bo = off; off += excp_pad16(8ull * excp_words((g.flags & 8u) ? n : nw));
            S.off_cw = off; off += excp_pad16(8ull * excp_words(nw * nb));
            S.off_cm = off; off += excp_pad16(8ull * excp_words(no * nb));
            S.off_cv = off; off += excp_pad16(8ull * excp_words(no * nb));
            S.blob_bytes = off;
            int status = 0;
            if (off > D.blob_cap) status = -2;
            if (S.nonfinite) status = -3;
            S.status = status;
        }
    }
    for (u32 q = 0; q < per; ++q) {
        u32 sidx = tid * per + q;
        if (sidx >= nseg) break;
        u32 t = sidx / 3u, which = sidx % 3u;
        TState &S = w.st[t];
        // the status is recomputed here: (t, 1) and (t, 2) may belong to another thread than (t, 0)
        u64 len = which == 0 ? S.n_w : S.n_o;
        const TDesc &D = w.desc[t];
        {
            const u64 n = D.n, nw = S.n_w, no = S.n_o, nb = (u64)g.nbits;
            u64 off = EXCP_HEADER + excp_books_bytes((u32)g.nbits) + excp_pad16(8ull * excp_words(n));
            off += excp_pad16(8ull * excp_words((g.flags & 8u) ? n : nw)) + excp_pad16(8ull * excp_words(nw * nb)) +
                   2ull * excp_pad16(8ull * excp_words(no * nb));
            if (off > D.blob_cap || S.nonfinite) len = 0;
        }
        w.seg[sidx].len = len;
        local += (u32)((len + EXCP_CHUNK - 1) / EXCP_CHUNK);
    }
    s_sum[tid] = local;
    __syncthreads();
    for (int off = 1; off < EXCP_THREADS; off <<= 1) {
        u32 v = (tid >= (u32)off) ? s_sum[tid - off] : 0u;
        __syncthreads();
        s_sum[tid] += v;
        __syncthreads();
    }
    u32 run = s_sum[tid] - local;
    for (u32 q = 0; q < per; ++q) {
        u32 sidx = tid * per + q;
        if (sidx >= nseg) break;
        seg_chunk_begin[sidx] = run;
        w.seg[sidx].chunk_begin = run;
        run += (u32)((w.seg[sidx].len + EXCP_CHUNK - 1) / EXCP_CHUNK);
    }
    if (tid == EXCP_THREADS - 1) { seg_chunk_begin[nseg] = s_sum[tid]; *w.chunk_total = s_sum[tid]; }
}

}  // namespace

void launch_mask_compact(const Workspace &w, const GroupParams &g, int phase, hipStream_t s) {
    if (!g.ntiles) return;
    const u32 nsub = 2u * g.ntiles;
    if (phase == 0) {
        u32 grid = excp_grid(w, 20);
        if (grid > nsub) grid = nsub;
        const bool nw2m = (g.flags & 8u) != 0, w16 = (g.flags & 0x30u) != 0;
        if (nw2m && w16) hipLaunchKernelGGL((k_mask_slots<true, true>), dim3(grid), dim3(EXCP_THREADS), 0, s, w, g);
        else if (nw2m) hipLaunchKernelGGL((k_mask_slots<true, false>), dim3(grid), dim3(EXCP_THREADS), 0, s, w, g);
        else if (w16) hipLaunchKernelGGL((k_mask_slots<false, true>), dim3(grid), dim3(EXCP_THREADS), 0, s, w, g);
        else hipLaunchKernelGGL((k_mask_slots<false, false>), dim3(grid), dim3(EXCP_THREADS), 0, s, w, g);
    } else if (phase == 1) {
        hipLaunchKernelGGL(k_mask_scan_parts, dim3(g.ntensors * MSCAN_PARTS), dim3(EXCP_THREADS), 0, s, w, g);
        hipLaunchKernelGGL(k_mask_scan, dim3(g.ntensors * MSCAN_PARTS), dim3(EXCP_THREADS), 0, s, w, g);
    } else {
        u32 grid = (nsub + 31) / 32;
        if (grid > excp_grid(w, 48)) grid = excp_grid(w, 48);
        hipLaunchKernelGGL(k_mask_gather, dim3(grid), dim3(EXCP_THREADS), 0, s, w, g);
        u32 grid_o = (g.ntiles + 3) / 4;
        if (grid_o > excp_grid(w, 16)) grid_o = excp_grid(w, 16);
        if (g.flags & 8u) hipLaunchKernelGGL(k_mask_bitmap_o_elems, dim3(grid_o), dim3(EXCP_THREADS), 0, s, w, g);
        else hipLaunchKernelGGL(k_mask_bitmap_o, dim3(grid_o), dim3(EXCP_THREADS), 0, s, w, g);
    }
}

void launch_layout(const Workspace &w, const GroupParams &g, hipStream_t s) {
    hipLaunchKernelGGL(k_layout, dim3(1), dim3(EXCP_THREADS), 0, s, w, g, w.seg_chunk_begin);
}
