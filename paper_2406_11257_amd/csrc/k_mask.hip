// Joint pruning masks (Sec. 3.2, Eq. "r_w" and Eq. "r_o") and the order-preserving compaction of
// the survivors.
//
// Pass A (k_mask_slots) reads W_prev, W_t, m and v once.  Work unit: a sub-tile of 2048 elements
// (half a 4096-element tile): 4 waves x 8 batches of 64, so that one wave ballot is one word of the
// keep bitmap.  It writes the keep bitmap, the sub-tile's survivor counts, and the survivors
// themselves -- compacted in index order, together with their M_o bits -- into the sub-tile's own
// slot of a scratch area.  No workgroup waits for another: where a survivor finally goes depends on
// the counts of all earlier sub-tiles, and that is left to a scan (k_mask_scan, one workgroup per
// tensor over its sub-tile counts) and to pass B (k_mask_gather), which copies every slot to its
// place in the dense survivor arrays; k_mask_bitmap_o then assembles bitmap_o from the sub-tiles'
// local bit streams.  The extra copy costs 8 bytes per survivor; it replaces a chained scan whose
// waits cost more than that.
#include <type_traits>

#include "excp_util.h"

namespace {

constexpr u32 SUB = 2048;          // elements per sub-tile
constexpr int NBATCH = 8;          // 64-element batches per wave and sub-tile
constexpr u32 BO_WORDS = SUB / 64; // M_o words kept per sub-tile

struct Regs {
    float w[NBATCH], p[NBATCH], m[NBATCH], v[NBATCH];
};

// sub-tile s of the group -> (tensor, first element); slots live in the partition arrays, which are
// free until the codebook stage
//
// NW2M (Table "vit", no weights-to-momentum check): M_o(i) = |m_i| > r_o for every element, kept
// weight or not.  The moment survivors are then compacted from the elements themselves, and the
// sub-tile's M_o words are indexed by element.
// W16: the two weight arrays hold 16-bit values (fp16 or bf16 by the flags), widened as they arrive.
template <bool NW2M, bool W16>
__global__ __launch_bounds__(EXCP_THREADS, 5) void k_mask_slots(Workspace w, GroupParams g) {
    __shared__ float l_w[SUB], l_m[SUB], l_v[SUB];      // compacted survivors of one sub-tile
    __shared__ u32 s_w[4], s_o[4];
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u64 lt_mask = lanemask_lt();
    const u32 nsub = 2u * g.ntiles;
    load_tile_table(s_tiles, w.tile_begin, g.ntensors);

    auto issue_loads = [&](u32 sub, Regs &R) {
        if (sub >= nsub) return;
        const u32 tile = sub >> 1;
        const u32 t = find_owner(s_tiles, g.ntensors, tile);
        const TDesc &D = w.desc[t];
        const u64 n = D.n;
        const u64 base = (u64)(tile - s_tiles[t]) * EXCP_TILE + (u64)(sub & 1u) * SUB;
        const bool bf = W16 && excp_wtype(g.flags) == 2u;
        if (base + SUB <= n) {
            // full sub-tile: one address per array and lane, the batches are immediate offsets
            const u64 first = base + (u64)(wave * (SUB / 4) + lane);
            const EXCP_GLOBAL float *gW = gptr(D.W) + first, *gP = gptr(D.Wp) + first;
            const EXCP_GLOBAL unsigned short *hW = gptr((const unsigned short *)D.W) + first;
            const EXCP_GLOBAL unsigned short *hP = gptr((const unsigned short *)D.Wp) + first;
            const EXCP_GLOBAL float *gM = gptr(D.m) + first, *gV = gptr(D.v) + first;
#pragma unroll
            for (int j = 0; j < NBATCH; ++j) {
                if (W16) { R.w[j] = w16_widen(hW[j * 64], bf); R.p[j] = w16_widen(hP[j * 64], bf); }
                else { R.w[j] = gW[j * 64]; R.p[j] = gP[j * 64]; }
                R.m[j] = gM[j * 64]; R.v[j] = gV[j * 64];
            }
        } else {
#pragma unroll
            for (int j = 0; j < NBATCH; ++j) {
                const u64 idx = base + (u64)((wave * NBATCH + j) * 64 + lane);
                const bool ok = idx < n;
                R.w[j] = ok ? load_weight(D.W, idx, W16 ? excp_wtype(g.flags) : 0u) : 0.f;
                R.p[j] = ok ? load_weight(D.Wp, idx, W16 ? excp_wtype(g.flags) : 0u) : 0.f;
                R.m[j] = ok ? D.m[idx] : 0.f;
                R.v[j] = ok ? D.v[idx] : 1.f;
            }
        }
    };

    auto compute = [&](u32 sub, Regs &R, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        const u32 tile = sub >> 1;
        const u32 t = find_owner(s_tiles, g.ntensors, tile);
        const TDesc &D = w.desc[t];
        const u64 n = D.n;
        const u32 first_sub = 2u * s_tiles[t];
        const u64 base = (u64)(sub - first_sub) * SUB;
        const float t_w = w.st[t].t_w, r_o = w.st[t].r_o;
        const u32 rem = FULL ? SUB : (u32)(n > base ? n - base : 0);      // valid elements here
        u64 bw[NBATCH];
        u32 nf = 0, cw = 0;
#pragma unroll
        for (int j = 0; j < NBATCH; ++j) {
            const u32 e = (wave * NBATCH + j) * 64 + lane;
            const bool ok = FULL || e < rem;
            R.w[j] = R.w[j] - R.p[j];                     // the residual
            // |d| > t_w / sqrt(v) with correctly rounded sqrt and divide, decided by a cheap estimate
            // when the estimate is not within 1e-5 of |d| (its own error is below 1e-6) and by the
            // exact expression otherwise, so the result is always that of the exact expression.
            // The estimate is trusted only for positive normal v and a positive normal estimate.
            const float ad = fabsf(R.w[j]);
            const float ra = t_w * __builtin_amdgcn_rsqf(R.v[j]);
            const bool sure_keep = ad > ra * 1.00001f, sure_drop = ad < ra * 0.99999f;
            const bool amb = !(sure_keep || sure_drop) || !__builtin_amdgcn_classf(R.v[j], 0x100) ||
                             !__builtin_amdgcn_classf(ra, 0x100);
            bool kw = sure_keep;
            if (g.flags & 2u) {
                kw = ad > t_w;                            // ablation: the same scalar threshold for every element
            } else if (__any(amb)) {
                // sqrtf and '/' are the correctly rounded forms (the build passes
                // -fhip-fp32-correctly-rounded-divide-sqrt); __fsqrt_rn is NOT on this target
                if (amb) kw = ad > t_w / sqrtf(R.v[j]);
            }
            kw = ok && kw;
            nf += ((f2u(R.v[j]) & 0x7f800000u) == 0x7f800000u);
            bw[j] = ballot64(kw);
            cw += __popcll(bw[j]);
        }
        // keep bitmap of the residual: one ballot per 64 elements
        {
            u64 *bm = (u64 *)(D.blob + EXCP_HEADER + excp_books_bytes((u32)g.nbits));
            const u64 nwords = excp_words(n);
            u64 mine = 0;
#pragma unroll
            for (int j = 0; j < NBATCH; ++j) if (lane == (u32)j) mine = bw[j];
            const u64 word = (base >> 6) + wave * NBATCH + lane;
            // words past the last element carry an all-zero ballot: that is the 16-byte padding
            if (lane < NBATCH && word < nwords + (nwords & 1ull)) bm[word] = mine;
        }
        nf = wave_sum_u32(nf);
        if (lane == 0) {
            s_w[wave] = cw;
            if (nf) atomicAdd(&w.st[t].nonfinite, (u64)nf);
        }
        __syncthreads();
        const u32 tw = s_w[0] + s_w[1] + s_w[2] + s_w[3];
        // compact the residual survivors (index order) in LDS, each with its M_o flag
        u32 pw = 0;
        for (u32 q = 0; q < wave; ++q) pw += s_w[q];
#pragma unroll
        for (int j = 0; j < NBATCH; ++j) {
            const u64 mw = bw[j];
            const bool kw = (mw >> lane) & 1ull;
            const u32 rk = pw + __popcll(mw & lt_mask);
            if (kw) {
                l_w[rk] = R.w[j];
                if (!NW2M) { l_m[rk] = R.m[j]; l_v[rk] = R.v[j]; }
            }
            pw += __popcll(mw);
        }
        __syncthreads();
        // second compaction, over the survivors: those whose moments are kept (M_o).  Survivor p
        // is handled by thread p % 256; a ballot over 64 consecutive survivors is one M_o word.
        const u64 slot = D.elem_off + base;
        EXCP_GLOBAL float *sw = gptr(w.pw) + slot, *sm = gptr(w.pm) + slot, *sv = gptr(w.pv) + slot;
        float mm[NBATCH], vv2[NBATCH]; u64 bo[NBATCH]; u32 co = 0;
#pragma unroll
        for (int j = 0; j < NBATCH; ++j) {
            const u32 p = (wave * NBATCH + j) * 64 + lane;       // survivor position in the sub-tile
            const bool in = p < tw;
            if (in) sw[p] = l_w[p];
            if (NW2M) {
                // p is also this lane's element of batch j
                mm[j] = R.m[j]; vv2[j] = R.v[j];
                bo[j] = ballot64((FULL || p < rem) && fabsf(mm[j]) > r_o);
            } else {
                mm[j] = in ? l_m[p] : 0.f;
                vv2[j] = in ? l_v[p] : 0.f;
                bo[j] = ballot64(in && fabsf(mm[j]) > r_o);
            }
            co += __popcll(bo[j]);
        }
        if (lane < NBATCH) {
            u64 mine = 0;
#pragma unroll
            for (int j = 0; j < NBATCH; ++j) if (lane == (u32)j) mine = bo[j];
            const u32 wordi = wave * NBATCH + lane;
            if (NW2M || wordi < ((tw + 63u) >> 6)) w.mask_bo[(u64)sub * BO_WORDS + wordi] = mine;
        }
        if (lane == 0) s_o[wave] = co;
        __syncthreads();
        const u32 to = s_o[0] + s_o[1] + s_o[2] + s_o[3];
        if (tid == 0) w.tile_status[sub] = ((u64)tw << 32) | (u64)to;
        u32 po = 0;
        for (u32 q = 0; q < wave; ++q) po += s_o[q];
#pragma unroll
        for (int j = 0; j < NBATCH; ++j) {
            const u64 mo = bo[j];
            if ((mo >> lane) & 1ull) {
                const u32 ro = po + __popcll(mo & lt_mask);
                sm[ro] = mm[j]; sv[ro] = vv2[j];
            }
            po += __popcll(mo);
        }
        __syncthreads();
    };

    auto sub_is_full = [&](u32 sub) -> bool {
        const u32 tile = sub >> 1;
        const u32 t = find_owner(s_tiles, g.ntensors, tile);
        const u64 base = (u64)(tile - s_tiles[t]) * EXCP_TILE + (u64)(sub & 1u) * SUB;
        return base + SUB <= w.desc[t].n;
    };
    Regs A;
    for (u32 sub = blockIdx.x; sub < nsub; sub += gridDim.x) {
        issue_loads(sub, A);
        if (sub_is_full(sub)) compute(sub, A, std::true_type{}); else compute(sub, A, std::false_type{});
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

// Pass B: one wave per sub-tile copies the slot to its place in the dense survivor arrays.  A workgroup takes 32
// consecutive sub-tiles; their counts, prefixes and tensor data are fetched once, side by side,
// into LDS, so that a wave's copies do not wait behind a chain of dependent look-ups.
constexpr u32 GATHER_SUBS = 32;

__global__ __launch_bounds__(EXCP_THREADS) void k_mask_gather(Workspace w, GroupParams g) {
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    __shared__ u32 s_tw[GATHER_SUBS], s_to[GATHER_SUBS], s_pw[GATHER_SUBS], s_po[GATHER_SUBS], s_t[GATHER_SUBS];
    __shared__ u64 s_slot[GATHER_SUBS], s_eoff[GATHER_SUBS];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 nsub = 2u * g.ntiles;
    load_tile_table(s_tiles, w.tile_begin, g.ntensors);
    for (u32 sub0 = blockIdx.x * GATHER_SUBS; sub0 < nsub; sub0 += gridDim.x * GATHER_SUBS) {
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
        for (u32 j = wave; j < GATHER_SUBS; j += 4) {
            const u32 tw = s_tw[j], to = s_to[j];
            if (tw == 0 && to == 0) continue;
            const u32 pw = s_pw[j], po = s_po[j];
            const u64 slot = s_slot[j], eoff = s_eoff[j];
            const EXCP_GLOBAL float *sw = gptr(w.pw) + slot, *sm = gptr(w.pm) + slot, *sv = gptr(w.pv) + slot;
            EXCP_GLOBAL float *xw = gptr(w.xw) + eoff + pw;
            EXCP_GLOBAL float *xm = gptr(w.xm) + eoff + po;
            EXCP_GLOBAL float *xv = gptr(w.xv) + eoff + po;
            {
                // the first batch of all three runs in flight together (usually there is no second)
                float qw[12], qm[4], qv[4];
                load_batch<12>(qw, sw, tw, 0, lane); load_batch<4>(qm, sm, to, 0, lane); load_batch<4>(qv, sv, to, 0, lane);
                store_batch<12>(xw, qw, tw, 0, lane); store_batch<4>(xm, qm, to, 0, lane); store_batch<4>(xv, qv, to, 0, lane);
                for (u32 b0 = 768u; b0 < tw; b0 += 768u) { load_batch<12>(qw, sw, tw, b0, lane); store_batch<12>(xw, qw, tw, b0, lane); }
                for (u32 b0 = 256u; b0 < to; b0 += 256u) {
                    load_batch<4>(qm, sm, to, b0, lane); load_batch<4>(qv, sv, to, b0, lane);
                    store_batch<4>(xm, qm, to, b0, lane); store_batch<4>(xv, qv, to, b0, lane);
                }
            }
        }
    }
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
