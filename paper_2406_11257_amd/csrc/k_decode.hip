// Reconstruction (Alg. 2): bitmap rank -> packed code -> codebook -> W_hat = W_prev + C_w[code],
// m_hat / v_hat = C[code] (zero where pruned).
//
// A tile of 4096 elements needs (a) the number of residual survivors before it, and (b) the number
// of moment survivors before its first residual survivor.  Both come from popcounts: per-tile
// counts of bitmap_w, an exclusive scan per tensor, then per-tile popcounts of the matching bit
// range of bitmap_o and a second scan.  The main pass is then independent per tile.
#include "excp_util.h"

namespace {

__device__ __forceinline__ u64 range_mask(u32 lo_bit, u32 hi_bit) {   // bits [lo_bit, hi_bit), hi_bit <= 64
    u64 hi = (hi_bit >= 64u) ? ~0ull : ((1ull << hi_bit) - 1ull);
    u64 lo = (lo_bit >= 64u) ? ~0ull : ((1ull << lo_bit) - 1ull);
    return hi & ~lo;
}

// popcount of bits [p0, p1) of a bitmap
__device__ __forceinline__ u32 popcount_range_lane(const u64 *__restrict__ bm, u64 p0, u64 p1, u32 lane) {
    // the calling wave covers up to 65 words: lane l takes word (p0 >> 6) + l, lane 0 also the 65th
    if (p1 <= p0) return 0;
    const u64 w0 = p0 >> 6, w1 = (p1 - 1) >> 6;
    u32 cnt = 0;
    for (u64 wi = w0 + lane; wi <= w1; wi += 64) {
        u64 word = bm[wi];
        u32 lo = (wi == w0) ? (u32)(p0 & 63ull) : 0u;
        u32 hi = (wi == w1) ? (u32)((p1 - 1) & 63ull) + 1u : 64u;
        cnt += __popcll(word & range_mask(lo, hi));
    }
    return cnt;
}

// Validate the header of every blob and derive the section offsets.
__global__ void k_decode_parse(Workspace w, u32 ntensors) {
    const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ntensors) return;
    const DDesc &D = w.ddesc[t];
    DState &S = w.dst[t];
    S.status = 0; S.pop_w = 0; S.pop_o = 0;
    S.n_w = 0; S.n_o = 0; S.nbits = 4; S.blob_bytes = 0;
    if (D.blob_bytes < EXCP_HEADER) { S.status = -4; return; }
    const u32 *h = (const u32 *)D.blob;
    const u64 *h64 = (const u64 *)D.blob;
    const u32 nbits = h[2];
    const u64 n = h64[2], nw = h64[3], no = h64[4], total = h64[8];
    bool ok = h[0] == EXCP_MAGIC && h[1] == EXCP_VERSION && nbits >= 2u && nbits <= 8u && h[3] == 0u;
    ok = ok && n == D.n && no <= nw && nw <= n;
    u64 off = EXCP_HEADER;
    if (ok) {
        off += 12ull * (1u << nbits);
        S.off_bw = off; off += excp_pad16(8ull * excp_words(n));
        S.off_bo = off; off += excp_pad16(8ull * excp_words(nw));
        S.off_cw = off; off += excp_pad16(8ull * excp_words(nw * nbits));
        S.off_cm = off; off += excp_pad16(8ull * excp_words(no * nbits));
        S.off_cv = off; off += excp_pad16(8ull * excp_words(no * nbits));
        ok = (off == total) && (total <= D.blob_bytes);
    }
    if (!ok) { S.status = -4; return; }
    S.n_w = nw; S.n_o = no; S.nbits = nbits; S.blob_bytes = total;
}

// which == 0: per-tile popcount of bitmap_w.  which == 1: per-tile popcount of the bitmap_o bits
// that belong to the tile's survivors (needs the scanned bitmap_w counts).  One wave per tile.
template <int WHICH>
__global__ __launch_bounds__(EXCP_THREADS) void k_decode_count(Workspace w, u32 ntensors, u32 ntiles) {
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    const u32 lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const u32 wpb = EXCP_THREADS / 64;
    load_tile_table(s_tiles, w.tile_begin, ntensors);
    for (u32 tile = blockIdx.x * wpb + wave; tile < ntiles; tile += gridDim.x * wpb) {
        const u32 t = find_owner(s_tiles, ntensors, tile);
        const DDesc &D = w.ddesc[t];
        const DState &S = w.dst[t];
        u32 cnt = 0;
        if (S.status == 0) {
            const u32 ltile = tile - D.tile_begin;
            if (WHICH == 0) {
                const u64 *bm = (const u64 *)(D.blob + S.off_bw);
                const u64 word = (u64)ltile * 64 + lane;
                if (word < excp_words(D.n)) {
                    u64 v = bm[word];
                    // bits beyond n must be clear in a well-formed blob; ignore them here
                    u64 rem = D.n - word * 64;
                    if (rem < 64) v &= (1ull << rem) - 1ull;
                    cnt = __popcll(v);
                }
            } else {
                const u64 *bm = (const u64 *)(D.blob + S.off_bo);
                u64 p0 = w.dec_cnt_w[tile];
                u64 p1 = (tile + 1 < D.tile_begin + D.tile_count) ? (u64)w.dec_cnt_w[tile + 1] : S.pop_w;
                if (p1 > S.n_w) p1 = S.n_w;          // damaged blob: stay inside the bitmap
                if (p0 > p1) p0 = p1;
                cnt = popcount_range_lane(bm, p0, p1, lane);
            }
            cnt = wave_sum_u32(cnt);
        }
        if (lane == 0) { if (WHICH == 0) w.dec_cnt_w[tile] = cnt; else w.dec_cnt_o[tile] = cnt; }
    }
}

// Exclusive scan of the per-tile counts of one tensor (one workgroup per tensor).
template <int WHICH>
__global__ __launch_bounds__(EXCP_THREADS) void k_decode_scan(Workspace w, u32 ntensors) {
    __shared__ u32 s_sum[EXCP_THREADS];
    const u32 t = blockIdx.x, tid = threadIdx.x;
    const DDesc &D = w.ddesc[t];
    DState &S = w.dst[t];
    u32 *cnt = (WHICH == 0 ? w.dec_cnt_w : w.dec_cnt_o) + D.tile_begin;
    u64 carry = 0;
    for (u32 base = 0; base < D.tile_count; base += EXCP_THREADS) {
        u32 i = base + tid;
        u32 v = (i < D.tile_count) ? cnt[i] : 0u;
        s_sum[tid] = v;
        __syncthreads();
        for (int off = 1; off < EXCP_THREADS; off <<= 1) {
            u32 a = (tid >= (u32)off) ? s_sum[tid - off] : 0u;
            __syncthreads();
            s_sum[tid] += a;
            __syncthreads();
        }
        if (i < D.tile_count) cnt[i] = (u32)(carry + s_sum[tid] - v);
        carry += s_sum[EXCP_THREADS - 1];
        __syncthreads();
    }
    if (tid == 0) {
        if (WHICH == 0) { S.pop_w = carry; if (S.status == 0 && carry != S.n_w) S.status = -4; }
        else { S.pop_o = carry; if (S.status == 0 && carry != S.n_o) S.status = -4; }
    }
}

// Code j of an nbits-wide little-endian bit stream.  Both words are always loaded (the second one
// clamped to the last word) so that no load sits behind a data-dependent branch.
__device__ __forceinline__ u32 extract_code(u64 w0, u64 w1, u32 sh, u32 nbits) {
    u64 v = w0 >> sh;
    if (sh) v |= w1 << (64u - sh);
    return (u32)(v & ((1ull << nbits) - 1ull));
}

template <bool MOMENTS>
__global__ __launch_bounds__(EXCP_THREADS) void k_decode_main(Workspace w, u32 ntensors, u32 ntiles) {
    __shared__ float s_book[3 * 256];
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u64 lt_mask = lanemask_lt();
    u32 cur_t = 0xffffffffu;
    load_tile_table(s_tiles, w.tile_begin, ntensors);
    for (u32 tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const u32 t = find_owner(s_tiles, ntensors, tile);
        const DDesc &D = w.ddesc[t];
        const DState &S = w.dst[t];
        if (S.status != 0) continue;
        const u32 nbits = S.nbits, E = 1u << nbits;
        if (t != cur_t) {
            __syncthreads();
            const float *books = (const float *)(D.blob + EXCP_HEADER);
            for (u32 i = tid; i < 3u * E; i += EXCP_THREADS) s_book[(i / E) * 256u + (i % E)] = books[i];
            cur_t = t;
            __syncthreads();
        }
        const u64 n = D.n;
        const u32 ltile = tile - D.tile_begin;
        const u64 base = (u64)ltile * EXCP_TILE;
        const float *__restrict__ Wp = D.Wp;
        const u64 *__restrict__ bmw = (const u64 *)(D.blob + S.off_bw);
        const u64 *__restrict__ bmo = (const u64 *)(D.blob + S.off_bo);
        const u64 *__restrict__ cw = (const u64 *)(D.blob + S.off_cw);
        const u64 *__restrict__ cm = (const u64 *)(D.blob + S.off_cm);
        const u64 *__restrict__ cv = (const u64 *)(D.blob + S.off_cv);
        const u64 nwords = excp_words(n);
        const u64 n_w = S.n_w, n_o = S.n_o;
        const bool pow2 = (64u % nbits) == 0u;
        const bool moments = MOMENTS && ((D.m_out != nullptr) || (D.v_out != nullptr));
        const bool inplace = D.W_out == D.Wp;

        // survivors before each of the tile's 64 bitmap words
        const u64 wword = (u64)ltile * 64 + lane;
        u64 myword = (wword < nwords) ? bmw[wword] : 0ull;
        {
            u64 rem = (wword * 64 < n) ? n - wword * 64 : 0ull;
            if (rem < 64) myword &= (1ull << rem) - 1ull;
        }
        u32 pc = __popcll(myword), incl = pc;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            u32 v = __shfl_up(incl, off, WAVE);
            if (lane >= (u32)off) incl += v;
        }
        const u32 excl = incl - pc;
        const u64 q_tile = w.dec_cnt_w[tile];          // survivors before this tile
        const u64 cw_last = n_w ? excp_words(n_w * nbits) - 1 : 0;

        // moments: prefix popcounts of the bitmap_o words that cover this tile's survivors
        const u64 o_tile = w.dec_cnt_o[tile];          // moment survivors before this tile
        const u64 ow0 = q_tile >> 6;
        const u64 nw_words = excp_words(n_w);
        u64 oword = 0, oword64 = 0; u32 oexcl = 0, ototal = 0;
        if (moments) {
            oword = (ow0 + lane < nw_words) ? bmo[ow0 + lane] : 0ull;
            oword64 = (ow0 + 64 < nw_words) ? bmo[ow0 + 64] : 0ull;
            u64 oword_m = oword;
            if (lane == 0) oword_m &= ~((1ull << (q_tile & 63ull)) - 1ull);   // bits before the tile's first survivor
            u32 opc = __popcll(oword_m), oincl = opc;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                u32 v = __shfl_up(oincl, off, WAVE);
                if (lane >= (u32)off) oincl += v;
            }
            oexcl = oincl - opc;
            ototal = __shfl(oincl, 63, WAVE);
        }
        const u64 cm_last = n_o ? excp_words(n_o * nbits) - 1 : 0;

        for (int half = 0; half < 2; ++half) {
            // ---- weights: all loads of eight batches first, then the arithmetic ----------------
            float wp[8]; u64 c0[8], c1[8]; u64 qq[8]; bool kwv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const u32 wi = wave * 16 + half * 8 + j;
                const u64 idx = base + (u64)(wi * 64 + lane);
                // wi is the same for the whole wave: a scalar lane read, no cross-lane permute
                const u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)myword, (int)wi);
                const u32 hi = (u32)__builtin_amdgcn_readlane((int)(u32)(myword >> 32), (int)wi);
                const u64 mw = ((u64)hi << 32) | lo;
                const u32 wexcl = (u32)__builtin_amdgcn_readlane((int)excl, (int)wi);
                const bool ok = idx < n;
                kwv[j] = ok && ((mw >> lane) & 1ull);
                u64 q = q_tile + wexcl + __popcll(mw & lt_mask);   // survivor position where kept
                if (q >= n_w) q = n_w ? n_w - 1 : 0;               // keeps every address in range
                qq[j] = q;
                wp[j] = Wp[ok ? idx : n - 1];
                const u64 wi0 = (q * nbits) >> 6;
                c0[j] = n_w ? cw[wi0] : 0ull;
                c1[j] = (!pow2 && n_w) ? cw[wi0 < cw_last ? wi0 + 1 : cw_last] : 0ull;
            }
            if (D.W_out) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const u64 idx = base + (u64)((wave * 16 + half * 8 + j) * 64 + lane);
                    const u32 code = extract_code(c0[j], c1[j], (u32)((qq[j] * nbits) & 63ull), nbits);
                    const float outw = kwv[j] ? wp[j] + s_book[code] : wp[j];
                    if (idx < n && (!inplace || kwv[j])) D.W_out[idx] = outw;
                }
            }
            if (!MOMENTS || !moments) continue;
            // ---- moments: M_o bit and rank of every survivor -----------------------------------
            bool kov[8]; u64 m0[8], m1[8], v0[8], v1[8]; u32 shv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const u64 q = qq[j];
                const u32 rel = (u32)((q >> 6) - ow0);             // 0..64 where kept
                const u32 src = rel & 63u;
                const u32 olo = __shfl((u32)oword, src, WAVE), ohi = __shfl((u32)(oword >> 32), src, WAVE);
                u32 opre = __shfl(oexcl, src, WAVE);
                u64 ow = ((u64)ohi << 32) | olo;
                if (rel >= 64u) { ow = oword64; opre = ototal; }
                const u32 bitpos = (u32)(q & 63ull);
                kov[j] = kwv[j] && ((ow >> bitpos) & 1ull);
                u64 below = ow & ((1ull << bitpos) - 1ull);
                if (rel == 0u) below &= ~((1ull << (q_tile & 63ull)) - 1ull);
                u64 qo = o_tile + opre + __popcll(below);
                if (qo >= n_o) qo = n_o ? n_o - 1 : 0;
                const u64 wi0 = (qo * nbits) >> 6;
                const u64 wi1 = wi0 < cm_last ? wi0 + 1 : cm_last;
                shv[j] = (u32)((qo * nbits) & 63ull);
                m0[j] = n_o ? cm[wi0] : 0ull;
                v0[j] = n_o ? cv[wi0] : 0ull;
                m1[j] = (!pow2 && n_o) ? cm[wi1] : 0ull;
                v1[j] = (!pow2 && n_o) ? cv[wi1] : 0ull;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const u64 idx = base + (u64)((wave * 16 + half * 8 + j) * 64 + lane);
                if (idx < n) {
                    const float outm = kov[j] ? s_book[256u + extract_code(m0[j], m1[j], shv[j], nbits)] : 0.f;
                    const float outv = kov[j] ? s_book[512u + extract_code(v0[j], v1[j], shv[j], nbits)] : 0.f;
                    if (D.m_out) D.m_out[idx] = outm;
                    if (D.v_out) D.v_out[idx] = outv;
                }
            }
        }
    }
}

__global__ void k_decode_finish(Workspace w, u32 ntensors, u32 rec_base) {
    const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ntensors) return;
    const DState &S = w.dst[t];
    HostRec &R = w.rec_dev[rec_base + t];
    R.n = w.ddesc[t].n; R.n_w = S.n_w; R.n_o = S.n_o; R.blob_bytes = S.blob_bytes; R.nonfinite = 0;
    R.abs_sum = 0.0; R.obj[0] = R.obj[1] = R.obj[2] = 0.0;
    R.med = R.mean32 = R.t_w = R.r_o = 0.f;
    R.status = S.status; R.pad = 0;
}

// Decode state for a blob the compress path has just written (no header parsing needed).
__global__ void k_decode_from_compress(Workspace w, GroupParams g) {
    const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= g.ntensors) return;
    const TDesc &C = w.desc[t];
    const TState &T = w.st[t];
    DDesc &D = w.ddesc[t];
    DState &S = w.dst[t];
    D.Wp = C.Wp; D.blob = C.blob; D.blob_bytes = T.blob_bytes; D.n = C.n;
    D.W_out = C.W_out; D.m_out = nullptr; D.v_out = nullptr;
    D.tile_begin = C.tile_begin; D.tile_count = C.tile_count;
    S.n_w = T.n_w; S.n_o = T.n_o; S.blob_bytes = T.blob_bytes; S.nbits = (u32)g.nbits;
    S.off_bw = EXCP_HEADER + 12ull * (1u << g.nbits);
    S.off_bo = T.off_bo; S.off_cw = T.off_cw; S.off_cm = T.off_cm; S.off_cv = T.off_cv;
    S.status = (T.status == 0 && C.W_out != nullptr) ? 0 : 1;    // 1 = skip silently
    S.pop_w = 0; S.pop_o = 0;
}

}  // namespace

void launch_decode_parse(const Workspace &w, u32 ntensors, hipStream_t s) {
    if (!ntensors) return;
    hipLaunchKernelGGL(k_decode_parse, dim3((ntensors + 255) / 256), dim3(256), 0, s, w, ntensors);
}
void launch_decode_from_compress(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_decode_from_compress, dim3((g.ntensors + 255) / 256), dim3(256), 0, s, w, g);
}
void launch_decode_count(const Workspace &w, u32 ntensors, u32 ntiles, int which, hipStream_t s) {
    if (!ntiles) return;
    u32 blocks = (ntiles + 3) / 4;
    if (blocks > 4096) blocks = 4096;
    if (which == 0) hipLaunchKernelGGL(k_decode_count<0>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
    else hipLaunchKernelGGL(k_decode_count<1>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
}
void launch_decode_scan(const Workspace &w, u32 ntensors, int which, hipStream_t s) {
    if (!ntensors) return;
    if (which == 0) hipLaunchKernelGGL(k_decode_scan<0>, dim3(ntensors), dim3(EXCP_THREADS), 0, s, w, ntensors);
    else hipLaunchKernelGGL(k_decode_scan<1>, dim3(ntensors), dim3(EXCP_THREADS), 0, s, w, ntensors);
}
void launch_decode_main(const Workspace &w, u32 ntensors, u32 ntiles, bool moments, hipStream_t s) {
    if (!ntiles) return;
    u32 blocks = ntiles < (u32)w.grid_stream * 4u ? ntiles : (u32)w.grid_stream * 4u;
    if (moments) hipLaunchKernelGGL(k_decode_main<true>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
    else hipLaunchKernelGGL(k_decode_main<false>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
}
void launch_decode_finish(const Workspace &w, u32 ntensors, hipStream_t s) {
    if (!ntensors) return;
    hipLaunchKernelGGL(k_decode_finish, dim3((ntensors + 255) / 256), dim3(256), 0, s, w, ntensors, w.rec_base);
}
