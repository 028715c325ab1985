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

// Which decoder takes a blob: 1 = codes and fp32 weights, 2 = codes and 16-bit weights, 4 = written
// without quantisation (either weight storage).
__device__ __forceinline__ u32 blob_kind(u32 nbits, u32 flags) {
    return nbits == EXCP_RAW_BITS ? 4u : (excp_wtype(flags) != 0u ? 2u : 1u);
}

__device__ __forceinline__ bool wants_moments(const DDesc &D) {
    return D.m_out != nullptr || D.v_out != nullptr || D.cm != nullptr || D.cv != nullptr;
}

// Validate the header of every blob and derive the section offsets.
__global__ void k_decode_parse(Workspace w, u32 ntensors, u32 allow_raw) {
    const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ntensors) return;
    const DDesc &D = w.ddesc[t];
    DState &S = w.dst[t];
    S.status = 0; S.pop_w = 0; S.pop_o = 0;
    S.n_w = 0; S.n_o = 0; S.nbits = 4; S.blob_bytes = 0; S.flags = 0; S.pad = 0;
    if (D.blob_bytes < EXCP_HEADER) { S.status = -4; return; }
    const u32 *h = (const u32 *)D.blob;
    const u64 *h64 = (const u64 *)D.blob;
    const u32 nbits = h[2];
    const u64 n = h64[2], nw = h64[3], no = h64[4], total = h64[8];
    const bool raw = (h[3] & 4u) != 0u;                   // written without quantisation: fp32 values, no codebooks
    const bool nw2m = (h[3] & 8u) != 0u;                  // bitmap_o over all elements, not over the kept residuals
    bool ok = h[0] == EXCP_MAGIC && h[1] == EXCP_VERSION && h[3] < 64u && (h[3] & 0x30u) != 0x30u;
    ok = ok && (raw ? (nbits == EXCP_RAW_BITS && allow_raw != 0u) : (nbits >= 2u && nbits <= 8u));
    ok = ok && n == D.n && nw <= n && no <= (nw2m ? n : nw);
    ok = ok && (D.wtype == 3u || D.wtype == excp_wtype(h[3]));      // the caller's arrays are what the blob expects
    u64 off = EXCP_HEADER;
    if (ok) {
        off += excp_books_bytes(nbits);
        S.off_bw = off; off += excp_pad16(8ull * excp_words(n));
        S.off_bo = off; off += excp_pad16(8ull * excp_words(nw2m ? n : nw));
        S.off_cw = off; off += excp_pad16(8ull * excp_words(nw * nbits));
        S.off_cm = off; off += excp_pad16(8ull * excp_words(no * nbits));
        S.off_cv = off; off += excp_pad16(8ull * excp_words(no * nbits));
        ok = (off == total) && (total <= D.blob_bytes);
    }
    if (!ok) { S.status = -4; return; }
    S.n_w = nw; S.n_o = no; S.nbits = nbits; S.blob_bytes = total; S.flags = h[3];
    atomicOr(w.dec_kinds, blob_kind(nbits, h[3]));
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
            } else if (wants_moments(D)) {                              // only where moments are wanted
                const u64 *bm = (const u64 *)(D.blob + S.off_bo);
                u64 p0 = w.dec_cnt_w[tile];
                u64 p1 = (tile + 1 < D.tile_begin + D.tile_count) ? (u64)w.dec_cnt_w[tile + 1] : S.pop_w;
                if (p1 > S.n_w) p1 = S.n_w;          // damaged blob: stay inside the bitmap
                if (p0 > p1) p0 = p1;
                if (S.flags & 8u) {                  // one bit per element: the tile's own range
                    p0 = (u64)ltile * EXCP_TILE;
                    p1 = (D.n - p0 < (u64)EXCP_TILE) ? D.n : p0 + EXCP_TILE;
                }
                cnt = popcount_range_lane(bm, p0, p1, lane);
            }
            cnt = wave_sum_u32(cnt);
        }
        if (lane == 0) { if (WHICH == 0) w.dec_cnt_w[tile] = cnt; else w.dec_cnt_o[tile] = cnt; }
    }
}

// Exclusive scan of the per-tile counts of every tensor.  A tensor's tiles are cut into sixteen parts,
// one workgroup each: first the parts' totals, then every workgroup scans its own part from the sum of
// the parts before it.
constexpr u32 DSCAN_PARTS = 16;

__device__ __forceinline__ void dscan_range(u32 ntiles, u32 part, u32 &s0, u32 &s1) {
    const u32 per = (ntiles + DSCAN_PARTS - 1u) / DSCAN_PARTS;
    s0 = min(part * per, ntiles);
    s1 = min(s0 + per, ntiles);
}

template <int WHICH>
__global__ __launch_bounds__(EXCP_THREADS) void k_decode_scan_parts(Workspace w, u32 ntensors) {
    __shared__ u64 s_sum[EXCP_THREADS / 64];
    const u32 t = blockIdx.x / DSCAN_PARTS, part = blockIdx.x % DSCAN_PARTS, tid = threadIdx.x;
    const DDesc &D = w.ddesc[t];
    if (WHICH == 1 && !wants_moments(D)) return;
    const u32 *cnt = (WHICH == 0 ? w.dec_cnt_w : w.dec_cnt_o) + D.tile_begin;
    u32 s0, s1;
    dscan_range(D.tile_count, part, s0, s1);
    u64 local = 0;
    for (u32 i = s0 + tid; i < s1; i += EXCP_THREADS) local += cnt[i];
    local = wave_sum_u64(local);
    if ((tid & 63u) == 0u) s_sum[tid >> 6] = local;
    __syncthreads();
    if (tid == 0) w.dec_part[(u64)t * DSCAN_PARTS + part] = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
}

template <int WHICH>
__global__ __launch_bounds__(EXCP_THREADS) void k_decode_scan(Workspace w, u32 ntensors) {
    __shared__ u32 s_sum[EXCP_THREADS];
    const u32 t = blockIdx.x / DSCAN_PARTS, part = blockIdx.x % DSCAN_PARTS, tid = threadIdx.x;
    const DDesc &D = w.ddesc[t];
    DState &S = w.dst[t];
    u32 *cnt = (WHICH == 0 ? w.dec_cnt_w : w.dec_cnt_o) + D.tile_begin;
    if (WHICH == 1 && !wants_moments(D)) return;    // bitmap_o is not used for this one
    u32 s0, s1;
    dscan_range(D.tile_count, part, s0, s1);
    u64 carry = 0;
    for (u32 q = 0; q < part; ++q) carry += w.dec_part[(u64)t * DSCAN_PARTS + q];
    if (part == DSCAN_PARTS - 1u && tid == 0) {
        const u64 total = carry + w.dec_part[(u64)t * DSCAN_PARTS + part];
        if (WHICH == 0) { S.pop_w = total; if (S.status == 0 && total != S.n_w) S.status = -4; }
        else { S.pop_o = total; if (S.status == 0 && total != S.n_o) S.status = -4; }
    }
    for (u32 base = s0; base < s1; base += EXCP_THREADS) {
        u32 i = base + tid;
        u32 v = (i < s1) ? cnt[i] : 0u;
        s_sum[tid] = v;
        __syncthreads();
        for (int off = 1; off < EXCP_THREADS; off <<= 1) {
            u32 a = (tid >= (u32)off) ? s_sum[tid - off] : 0u;
            __syncthreads();
            s_sum[tid] += a;
            __syncthreads();
        }
        if (i < s1) cnt[i] = (u32)(carry + s_sum[tid] - v);
        carry += s_sum[EXCP_THREADS - 1];
        __syncthreads();
    }
}

// Four consecutive floats at an address that is only known to be 4-byte aligned.
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

#define DEC_CODE_WORDS 1032   // u32 words of one tile's codes: 4096 codes x 8 bits / 32 + slack
#define DEC_OBIT_WORDS 136    // u32 words of bitmap_o covering one tile's survivors: 4096 / 32 + slack

// Stage u32 words [first, first + count) of a blob section into LDS.
__device__ __forceinline__ void stage_words(u32 *dst, const EXCP_GLOBAL u32 *src, u32 count) {
    for (u32 i = threadIdx.x; i < count; i += EXCP_THREADS) dst[i] = src[i];
}

// 32 stream bits starting at bit p of a staged word array (p / 32 + 1 must be inside the array).
__device__ __forceinline__ u32 window32(const u32 *s, u32 p) {
    const u32 i = p >> 5;
    return __builtin_amdgcn_alignbit(s[i + 1], s[i], p & 31u);
}

// The codes of four consecutive elements (the first has index e0, a multiple of 4; `left` of them
// exist) into a per-element code tensor: half a byte each when nbits <= 4, else a byte each.
__device__ __forceinline__ void store_codes4(unsigned char *dst, u64 e0, u32 left, u32 nbits, const u32 c[4]) {
    if (left == 0u) return;
    if (nbits <= 4u) {
        const u32 v = c[0] | (c[1] << 4) | (c[2] << 8) | (c[3] << 12);
        EXCP_GLOBAL unsigned char *p = gptr(dst) + (e0 >> 1);
        if (left > 2u) *(EXCP_GLOBAL unsigned short *)p = (unsigned short)v;
        else *p = (unsigned char)v;
    } else {
        const u32 v = c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24);
        EXCP_GLOBAL unsigned char *p = gptr(dst) + e0;
        if (left >= 4u) *(EXCP_GLOBAL u32 *)p = v;
        else for (u32 j = 0; j < left; ++j) p[j] = (unsigned char)(v >> (8u * j));
    }
}

// One tile (4096 elements) per workgroup iteration.  Each wave scans the tile's 64 bitmap words,
// the workgroup stages the tile's contiguous run of packed codes (and, for the moments, the run of
// bitmap_o bits of its survivors with their prefix counts) in LDS, then every lane reconstructs four
// consecutive elements: the codes of its survivors are consecutive fields of the staged stream, so
// one 32-bit window read per lane holds all of them.
//
// DENSE: the same walk writes, instead of the reconstructed values, the codes themselves as the
// per-element code tensors of Sec. 4.2 (0 where pruned; two codes per byte when nbits <= 4, the
// even element in the low four bits; one code per byte otherwise).
//
// RAW: blobs written without quantisation hold fp32 values where the others hold codes; a lane reads
// its survivors' values straight from the blob (consecutive lanes, consecutive addresses).  Such
// blobs are skipped by the other instantiations, and this one skips everything else.
//
// WMODE: which weight storage this instantiation takes (blob flags bits 4-5): 0 = fp32 blobs only,
// 1 = blobs of 16-bit weights only (fp16 / bf16: widened exactly, the sum rounded to nearest even
// into the format, pruned positions keep their bits), 2 = both, decided per tensor.
template <bool MOMENTS, bool DENSE, bool RAW, int WMODE>
__device__ __forceinline__ void decode_tiles(const Workspace &w, u32 ntensors, u32 ntiles) {
    __shared__ float s_book[DENSE || RAW ? 1 : 3 * 256];
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    __shared__ u32 s_cw[RAW ? 2 : DEC_CODE_WORDS];
    __shared__ u32 s_cm[MOMENTS && !RAW ? DEC_CODE_WORDS : 2], s_cv[MOMENTS && !RAW ? DEC_CODE_WORDS : 2];
    __shared__ u32 s_ow[MOMENTS ? DEC_OBIT_WORDS : 1], s_oex[MOMENTS ? DEC_OBIT_WORDS : 1];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    u32 cur_t = 0xffffffffu;
    load_tile_table(s_tiles, w.tile_begin, ntensors);
    for (u32 tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const u32 t = find_owner(s_tiles, ntensors, tile);
        const DDesc &D = w.ddesc[t];
        const DState &S = w.dst[t];
        if (S.status != 0) continue;                       // same decision for the whole workgroup
        if ((S.nbits == EXCP_RAW_BITS) != RAW) continue;
        const u32 wt = WMODE == 0 ? 0u : excp_wtype(S.flags);
        if (WMODE == 0 && excp_wtype(S.flags) != 0u) continue;
        if (WMODE == 1 && wt == 0u) continue;
        const bool bf = wt == 2u;
        const u32 nbits = S.nbits, E = RAW ? 0u : 1u << (nbits & 15u), cmask = E - 1u;
        const u64 n = D.n;
        const u32 ltile = tile - D.tile_begin;
        const u64 base = (u64)ltile * EXCP_TILE;
        const u32 rem = (n - base < (u64)EXCP_TILE) ? (u32)(n - base) : EXCP_TILE;   // elements of this tile
        const unsigned char *blob = D.blob;
        const bool has_w = DENSE ? D.cw != nullptr : D.W_out != nullptr;
        const bool has_m = MOMENTS && (DENSE ? D.cm != nullptr : D.m_out != nullptr);
        const bool has_v = MOMENTS && (DENSE ? D.cv != nullptr : D.v_out != nullptr);
        const bool moments = has_m || has_v;
        if (!has_w && !moments) continue;                  // nothing to write for this one

        // previous weights of the lane's 4 x 4 elements: issued first, consumed last
        float wp[4][4];
        us4 hp[4];                                         // 16-bit weights stay as they are until the sum
        if (!DENSE && has_w && WMODE != 0 && wt != 0u) {
            const EXCP_GLOBAL unsigned short *Hp = gptr((const unsigned short *)D.Wp) + base;
            const bool vec = ((uintptr_t)D.Wp & 7u) == 0u;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u32 off = wave * 1024u + (u32)k * 256u + lane * 4u;
                if (vec && off + 4u <= rem) hp[k] = *(const EXCP_GLOBAL us4 *)(Hp + off);
                else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) hp[k][j] = (off + (u32)j < rem) ? Hp[off + (u32)j] : (unsigned short)0;
                }
            }
        } else if (!DENSE && has_w) {
            const EXCP_GLOBAL float *Wp = gptr(D.Wp) + base;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u32 off = wave * 1024u + (u32)k * 256u + lane * 4u;
                if (off + 4u <= rem) {
                    const f4u x = *(const EXCP_GLOBAL f4u *)(Wp + off);
                    wp[k][0] = x.x; wp[k][1] = x.y; wp[k][2] = x.z; wp[k][3] = x.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) wp[k][j] = (off + (u32)j < rem) ? Wp[off + (u32)j] : 0.f;
                }
            }
        }

        // survivors before each of the tile's 64 bitmap words (every wave computes all 64)
        u64 myword = 0;
        {
            const u64 wword = (u64)ltile * 64 + lane;
            const u32 bits_here = (lane * 64u < rem) ? min(64u, rem - lane * 64u) : 0u;
            if (bits_here) myword = gptr((const u64 *)(blob + S.off_bw))[wword];
            if (bits_here < 64u) myword &= (1ull << bits_here) - 1ull;
        }
        const u32 pc = __popcll(myword);
        u32 incl = pc;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const u32 v = __shfl_up(incl, off, WAVE);
            if (lane >= (u32)off) incl += v;
        }
        const u32 excl = incl - pc;
        const u32 cnt = __shfl(incl, 63, WAVE);            // survivors of this tile
        const u32 q_tile = w.dec_cnt_w[tile];              // survivors before this tile
        const u64 wbit0 = (u64)q_tile * nbits;
        const u32 woff = (u32)(wbit0 & 31ull);
        u32 o_tile = 0, ocnt = 0, moff = 0, ooff = 0;
        const bool nw2m = MOMENTS && (S.flags & 8u) != 0u;    // M_o bits per element instead of per kept residual
        if (MOMENTS && moments) {
            o_tile = w.dec_cnt_o[tile];
            const u32 o_next = (ltile + 1u < D.tile_count) ? w.dec_cnt_o[tile + 1] : (u32)S.pop_o;
            ocnt = o_next - o_tile;
            moff = (u32)(((u64)o_tile * nbits) & 31ull);
            ooff = nw2m ? 0u : q_tile & 31u;
        }

        __syncthreads();                                   // the previous tile's LDS readers are done
        if (!DENSE && !RAW && t != cur_t) {
            const EXCP_GLOBAL float *books = gptr((const float *)(blob + EXCP_HEADER));
            for (u32 i = tid; i < 3u * E; i += EXCP_THREADS) s_book[(i / E) * 256u + (i % E)] = books[i];
            cur_t = t;
        }
        if (!RAW) stage_words(s_cw, gptr((const u32 *)(blob + S.off_cw)) + (wbit0 >> 5), (woff + cnt * nbits + 31u) >> 5);
        if (MOMENTS && moments) {
            const u64 mbit0 = (u64)o_tile * nbits;
            const u32 mwords = (moff + ocnt * nbits + 31u) >> 5;
            if (!RAW) {
                stage_words(s_cm, gptr((const u32 *)(blob + S.off_cm)) + (mbit0 >> 5), mwords);
                stage_words(s_cv, gptr((const u32 *)(blob + S.off_cv)) + (mbit0 >> 5), mwords);
            }
            if (wave == 0) {
                // bitmap_o bits [q_tile, q_tile + cnt) as u32 words, with the count of set bits before each word
                const EXCP_GLOBAL u32 *bo = gptr((const u32 *)(blob + S.off_bo)) + (nw2m ? ltile * (EXCP_TILE / 32u) : q_tile >> 5);
                const u32 obits_total = nw2m ? rem : ooff + cnt;
                const u32 owords = (obits_total + 31u) >> 5;       // <= 129
                u32 carry = 0;
#pragma unroll
                for (int c = 0; c < 3; ++c) {
                    const u32 i = lane + 64u * (u32)c;
                    u32 word = (i < owords) ? bo[i] : 0u;
                    if (i == 0u) word &= ~((1u << ooff) - 1u);     // bits of earlier tiles' survivors
                    if (nw2m && i + 1u == owords && (obits_total & 31u)) word &= (1u << (obits_total & 31u)) - 1u;   // bits past the last element
                    const u32 opc = __popc(word);
                    u32 oincl = opc;
#pragma unroll
                    for (int off = 1; off < 64; off <<= 1) {
                        const u32 v = __shfl_up(oincl, off, WAVE);
                        if (lane >= (u32)off) oincl += v;
                    }
                    if (i < DEC_OBIT_WORDS) { s_ow[i] = word; s_oex[i] = carry + oincl - opc; }
                    carry += __shfl(oincl, 63, WAVE);
                }
            }
        }
        __syncthreads();

#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const u32 off = wave * 1024u + (u32)k * 256u + lane * 4u;   // first of the lane's 4 elements
            const u32 wq = wave * 16u + (u32)k * 4u + (lane >> 4);       // their bitmap word
            const u32 sub = (lane & 15u) * 4u;                           // their first bit in it
            const u32 wlo = __shfl((u32)myword, wq, WAVE), whi = __shfl((u32)(myword >> 32), wq, WAVE);
            const u32 wex = __shfl(excl, wq, WAVE);
            const u64 word = ((u64)whi << 32) | wlo;
            const u32 nib = (u32)(word >> sub) & 15u;
            const u32 r = wex + __popcll(word & ((1ull << sub) - 1ull));   // tile rank of the lane's first survivor
            u32 f = RAW ? 0u : window32(s_cw, woff + r * nbits);
            const EXCP_GLOBAL float *xw = gptr((const float *)(blob + S.off_cw)) + q_tile + r;   // RAW: the lane's first survivor
            if (DENSE) {
                if (has_w) {
                    u32 c[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const bool kept = (nib >> j) & 1u;
                        c[j] = kept ? (f & cmask) : 0u;
                        f = kept ? (f >> nbits) : f;
                    }
                    store_codes4(D.cw, base + off, rem - min(rem, off), nbits, c);
                }
            } else if (has_w && WMODE != 0 && wt != 0u) {
                us4 o16;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool kept = (nib >> j) & 1u;
                    float c;
                    if (RAW) { c = kept ? *xw : 0.f; xw += kept; }
                    else c = s_book[f & cmask];
                    const u32 h = hp[k][j];
                    o16[j] = (unsigned short)(kept ? w16_narrow(w16_widen(h, bf) + c, bf) : h);
                    f = kept ? (f >> nbits) : f;
                }
                EXCP_GLOBAL unsigned short *Ho = gptr((unsigned short *)D.W_out) + base;
                if (((uintptr_t)D.W_out & 7u) == 0u && off + 4u <= rem) *(EXCP_GLOBAL us4 *)(Ho + off) = o16;
                else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) if (off + (u32)j < rem) Ho[off + (u32)j] = o16[j];
                }
            } else if (has_w) {
                float out[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool kept = (nib >> j) & 1u;
                    float c;
                    if (RAW) { c = kept ? *xw : 0.f; xw += kept; }
                    else c = s_book[f & cmask];
                    out[j] = kept ? wp[k][j] + c : wp[k][j];
                    f = kept ? (f >> nbits) : f;
                }
                EXCP_GLOBAL float *Wo = gptr(D.W_out) + base;
                if (off + 4u <= rem) {
                    f4u y; y.x = out[0]; y.y = out[1]; y.z = out[2]; y.w = out[3];
                    *(EXCP_GLOBAL f4u *)(Wo + off) = y;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) if (off + (u32)j < rem) Wo[off + (u32)j] = out[j];
                }
            }
            if (MOMENTS && moments) {
                const u32 bpos = nw2m ? off : ooff + r;                   // the first survivor's (element's) bit in the staged bitmap_o
                const u32 bi = bpos >> 5, bsh = bpos & 31u;
                u32 obits = __builtin_amdgcn_alignbit(s_ow[bi + 1], s_ow[bi], bsh);
                const u32 orank = s_oex[bi] + __popc(s_ow[bi] & ((1u << bsh) - 1u));
                u32 fm = RAW ? 0u : window32(s_cm, moff + orank * nbits);
                u32 fv = RAW ? 0u : window32(s_cv, moff + orank * nbits);
                const EXCP_GLOBAL float *xm = gptr((const float *)(blob + S.off_cm)) + o_tile + orank;   // RAW
                const EXCP_GLOBAL float *xv = gptr((const float *)(blob + S.off_cv)) + o_tile + orank;
                if (DENSE) {
                    u32 cm4[4], cv4[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const bool kept = (nib >> j) & 1u;
                        const bool ko = (kept || nw2m) && (obits & 1u);
                        cm4[j] = ko ? (fm & cmask) : 0u;
                        cv4[j] = ko ? (fv & cmask) : 0u;
                        obits = (kept || nw2m) ? (obits >> 1) : obits;
                        fm = ko ? (fm >> nbits) : fm;
                        fv = ko ? (fv >> nbits) : fv;
                    }
                    if (has_m) store_codes4(D.cm, base + off, rem - min(rem, off), nbits, cm4);
                    if (has_v) store_codes4(D.cv, base + off, rem - min(rem, off), nbits, cv4);
                    continue;
                }
                float om[4], ov[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool kept = (nib >> j) & 1u;
                    const bool ko = (kept || nw2m) && (obits & 1u);
                    if (RAW) {
                        om[j] = ko ? *xm : 0.f; ov[j] = ko ? *xv : 0.f;
                        xm += ko; xv += ko;
                    } else {
                        om[j] = ko ? s_book[256u + (fm & cmask)] : 0.f;
                        ov[j] = ko ? s_book[512u + (fv & cmask)] : 0.f;
                    }
                    obits = (kept || nw2m) ? (obits >> 1) : obits;
                    fm = ko ? (fm >> nbits) : fm;
                    fv = ko ? (fv >> nbits) : fv;
                }
                if (off + 4u <= rem) {
                    f4u y;
                    if (has_m) { y.x = om[0]; y.y = om[1]; y.z = om[2]; y.w = om[3]; *(EXCP_GLOBAL f4u *)(gptr(D.m_out) + base + off) = y; }
                    if (has_v) { y.x = ov[0]; y.y = ov[1]; y.z = ov[2]; y.w = ov[3]; *(EXCP_GLOBAL f4u *)(gptr(D.v_out) + base + off) = y; }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (off + (u32)j < rem) {
                            if (has_m) gptr(D.m_out)[base + off + (u32)j] = om[j];
                            if (has_v) gptr(D.v_out)[base + off + (u32)j] = ov[j];
                        }
                    }
                }
            }
        }
    }
}

template <bool MOMENTS>
__global__ __launch_bounds__(EXCP_THREADS, MOMENTS ? 6 : 8) void k_decode_main(Workspace w, u32 ntensors, u32 ntiles) {
    if ((*w.dec_kinds & 1u) == 0u) return;                 // no blob of fp32 weights in this group
    decode_tiles<MOMENTS, false, false, 0>(w, ntensors, ntiles);
}
// The same for blobs of 16-bit weights (most batches hold none).
template <bool MOMENTS>
__global__ __launch_bounds__(EXCP_THREADS, MOMENTS ? 6 : 8) void k_decode_main16(Workspace w, u32 ntensors, u32 ntiles) {
    if ((*w.dec_kinds & 2u) == 0u) return;
    decode_tiles<MOMENTS, false, false, 1>(w, ntensors, ntiles);
}
// Blobs written without quantisation (most batches hold none).
template <bool MOMENTS>
__global__ __launch_bounds__(EXCP_THREADS) void k_decode_raw(Workspace w, u32 ntensors, u32 ntiles) {
    if ((*w.dec_kinds & 4u) == 0u) return;
    decode_tiles<MOMENTS, false, true, 2>(w, ntensors, ntiles);
}
template <bool MOMENTS>
__global__ __launch_bounds__(EXCP_THREADS, 8) void k_export_dense(Workspace w, u32 ntensors, u32 ntiles) {
    decode_tiles<MOMENTS, true, false, 2>(w, ntensors, ntiles);
}

// Alg. 3: W_0 plus a chain of compressed checkpoints, oldest first, in ONE pass over the weights.
// A lane keeps its sixteen weights in registers and adds, checkpoint after checkpoint, the centre
// of every kept element (one fp32 addition per checkpoint, exactly what applying Alg. 2 again and
// again computes); W_0 is read once and the result written once, whatever the length of the chain.
__global__ __launch_bounds__(EXCP_THREADS, 8) void k_decode_chain(Workspace w, u32 ntensors, u32 ntiles) {
    __shared__ float s_book[256];
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    __shared__ u32 s_cw[DEC_CODE_WORDS];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    load_tile_table(s_tiles, w.chain_tile_begin, ntensors);
    for (u32 tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const u32 t = find_owner(s_tiles, ntensors, tile);
        const CDesc &C = w.cdesc[t];
        if (C.W_out == nullptr) continue;
        bool good = true;                                  // every checkpoint of the chain parsed and counted fine
        const u32 wt = excp_wtype(w.dst[C.first_desc].flags);      // ... and all store their weights alike
        for (u32 j = 0; j < C.steps; ++j)
            good = good && w.dst[C.first_desc + j].status == 0 && excp_wtype(w.dst[C.first_desc + j].flags) == wt;
        if (!good) continue;                               // same decision for the whole workgroup
        const bool bf = wt == 2u;
        const u64 n = C.n;
        const u32 ltile = tile - C.tile_begin;
        const u64 base = (u64)ltile * EXCP_TILE;
        const u32 rem = (n - base < (u64)EXCP_TILE) ? (u32)(n - base) : EXCP_TILE;
        float wp[4][4];
        if (wt == 0u) {
            const EXCP_GLOBAL float *W0 = gptr(C.W0) + base;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u32 off = wave * 1024u + (u32)k * 256u + lane * 4u;
                if (off + 4u <= rem) {
                    const f4u x = *(const EXCP_GLOBAL f4u *)(W0 + off);
                    wp[k][0] = x.x; wp[k][1] = x.y; wp[k][2] = x.z; wp[k][3] = x.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) wp[k][j] = (off + (u32)j < rem) ? W0[off + (u32)j] : 0.f;
                }
            }
        }
        if (wt != 0u) {                                    // 16-bit weights: the registers hold the widened values
#pragma unroll
            for (int k = 0; k < 4; ++k) load_weights4(C.W0, base, wave * 1024u + (u32)k * 256u + lane * 4u, rem, wt, wp[k]);
        }
        for (u32 step = 0; step < C.steps; ++step) {
            const DDesc &D = w.ddesc[C.first_desc + step];
            const DState &S = w.dst[C.first_desc + step];
            const u32 nbits = S.nbits, E = 1u << nbits, cmask = E - 1u;
            const unsigned char *blob = D.blob;
            u64 myword = 0;
            {
                const u64 wword = (u64)ltile * 64 + lane;
                const u32 bits_here = (lane * 64u < rem) ? min(64u, rem - lane * 64u) : 0u;
                if (bits_here) myword = gptr((const u64 *)(blob + S.off_bw))[wword];
                if (bits_here < 64u) myword &= (1ull << bits_here) - 1ull;
            }
            const u32 pc = __popcll(myword);
            u32 incl = pc;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const u32 v = __shfl_up(incl, off, WAVE);
                if (lane >= (u32)off) incl += v;
            }
            const u32 excl = incl - pc;
            const u32 cnt = __shfl(incl, 63, WAVE);
            const u32 q_tile = w.dec_cnt_w[D.tile_begin + ltile];
            const u64 wbit0 = (u64)q_tile * nbits;
            const u32 woff = (u32)(wbit0 & 31ull);
            __syncthreads();                               // the previous checkpoint's LDS readers are done
            {
                const EXCP_GLOBAL float *book = gptr((const float *)(blob + EXCP_HEADER));
                for (u32 i = tid; i < E; i += EXCP_THREADS) s_book[i] = book[i];
            }
            stage_words(s_cw, gptr((const u32 *)(blob + S.off_cw)) + (wbit0 >> 5), (woff + cnt * nbits + 31u) >> 5);
            __syncthreads();
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u32 wq = wave * 16u + (u32)k * 4u + (lane >> 4);
                const u32 sub = (lane & 15u) * 4u;
                const u32 wlo = __shfl((u32)myword, wq, WAVE), whi = __shfl((u32)(myword >> 32), wq, WAVE);
                const u32 wex = __shfl(excl, wq, WAVE);
                const u64 word = ((u64)whi << 32) | wlo;
                const u32 nib = (u32)(word >> sub) & 15u;
                const u32 r = wex + __popcll(word & ((1ull << sub) - 1ull));
                u32 f = window32(s_cw, woff + r * nbits);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool kept = (nib >> j) & 1u;
                    const float c = s_book[f & cmask];
                    float sum = wp[k][j] + c;
                    if (wt != 0u) sum = w16_widen(w16_narrow(sum, bf), bf);   // every checkpoint rounds into the storage format
                    wp[k][j] = kept ? sum : wp[k][j];
                    f = kept ? (f >> nbits) : f;
                }
            }
        }
        if (wt != 0u) {
            EXCP_GLOBAL unsigned short *Ho = gptr((unsigned short *)C.W_out) + base;
            const bool vec = ((uintptr_t)C.W_out & 7u) == 0u;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u32 off = wave * 1024u + (u32)k * 256u + lane * 4u;
                us4 o16;
#pragma unroll
                for (int j = 0; j < 4; ++j) o16[j] = (unsigned short)w16_narrow(wp[k][j], bf);
                if (vec && off + 4u <= rem) *(EXCP_GLOBAL us4 *)(Ho + off) = o16;
                else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) if (off + (u32)j < rem) Ho[off + (u32)j] = o16[j];
                }
            }
            continue;
        }
        EXCP_GLOBAL float *Wo = gptr(C.W_out) + base;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const u32 off = wave * 1024u + (u32)k * 256u + lane * 4u;
            if (off + 4u <= rem) {
                f4u y; y.x = wp[k][0]; y.y = wp[k][1]; y.z = wp[k][2]; y.w = wp[k][3];
                *(EXCP_GLOBAL f4u *)(Wo + off) = y;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) if (off + (u32)j < rem) Wo[off + (u32)j] = wp[k][j];
            }
        }
    }
}

// Per tensor of a chain: status = the first checkpoint that failed, counts and size of the last one.
__global__ void k_chain_finish(Workspace w, u32 ntensors, u32 rec_base) {
    const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ntensors) return;
    const CDesc &C = w.cdesc[t];
    int status = 0;
    for (u32 j = 0; j < C.steps && status == 0; ++j) {
        status = w.dst[C.first_desc + j].status;
        if (status == 0 && excp_wtype(w.dst[C.first_desc + j].flags) != excp_wtype(w.dst[C.first_desc].flags)) status = -4;
    }
    const DState &S = w.dst[C.first_desc + C.steps - 1u];
    HostRec &R = w.rec_dev[rec_base + t];
    R.n = C.n; R.n_w = S.n_w; R.n_o = S.n_o; R.blob_bytes = S.blob_bytes; R.nonfinite = 0;
    R.abs_sum = 0.0; R.obj[0] = R.obj[1] = R.obj[2] = 0.0;
    R.med = R.mean32 = R.t_w = R.r_o = 0.f;
    R.status = status; R.pad = 0;
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

// Export: header and codebooks of every well-formed blob, verbatim (one workgroup per tensor).
__global__ void k_export_head(Workspace w, u32 ntensors) {
    const u32 t = blockIdx.x;
    const DDesc &D = w.ddesc[t];
    const DState &S = w.dst[t];
    if (S.status != 0 || D.head == nullptr) return;
    const u32 words = (EXCP_HEADER + 12u * (1u << S.nbits)) / 4u;
    const EXCP_GLOBAL u32 *src = gptr((const u32 *)D.blob);
    EXCP_GLOBAL u32 *dst = gptr((u32 *)D.head);
    for (u32 i = threadIdx.x; i < words; i += blockDim.x) dst[i] = src[i];
}

// Reconstruction from the per-element code tensors: here `blob` holds only header and codebooks.
__global__ void k_dense_parse(Workspace w, u32 ntensors) {
    const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ntensors) return;
    const DDesc &D = w.ddesc[t];
    DState &S = w.dst[t];
    S.status = 0; S.pop_w = 0; S.pop_o = 0;
    S.n_w = 0; S.n_o = 0; S.nbits = 4; S.blob_bytes = 0; S.flags = 0; S.pad = 0;
    if (D.blob_bytes < EXCP_HEADER) { S.status = -4; return; }
    const u32 *h = (const u32 *)D.blob;
    const u64 *h64 = (const u64 *)D.blob;
    const u32 nbits = h[2];
    bool ok = h[0] == EXCP_MAGIC && h[1] == EXCP_VERSION && nbits >= 2u && nbits <= 8u && h[3] < 64u && (h[3] & 0x30u) != 0x30u;
    ok = ok && h64[2] == D.n && D.blob_bytes >= EXCP_HEADER + 12ull * (1u << (nbits & 15u));
    ok = ok && (D.wtype == 3u || D.wtype == excp_wtype(h[3]));
    if (!ok) { S.status = -4; return; }
    S.n_w = h64[3]; S.n_o = h64[4]; S.nbits = nbits; S.blob_bytes = h64[8]; S.flags = h[3];
}

// Eight consecutive elements per lane and step: one 32-bit (or 64-bit) load of codes per tensor,
// two 16-byte loads of the previous weights, two 16-byte stores per output.  Code 0 leaves the
// weight untouched (not "+ 0.0": a negative zero stays) and gives a zero moment.  A code beyond the
// codebook, or a set unused half of the last byte, marks the tensor as damaged.
__global__ __launch_bounds__(EXCP_THREADS) void k_decode_dense(Workspace w, u32 ntensors, u32 ntiles) {
    __shared__ float s_book[3 * 256];
    __shared__ u32 s_tiles[EXCP_MAX_GROUP_TENSORS + 1];
    const u32 tid = threadIdx.x;
    u32 cur_t = 0xffffffffu;
    load_tile_table(s_tiles, w.tile_begin, ntensors);
    for (u32 tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const u32 t = find_owner(s_tiles, ntensors, tile);
        const DDesc &D = w.ddesc[t];
        DState &S = w.dst[t];
        if (S.status != 0 && S.status != -40) continue;    // -40: damage found by another workgroup meanwhile
        const u32 nbits = S.nbits, E = 1u << nbits;
        const bool wide = nbits > 4u;
        const u32 wt = excp_wtype(S.flags);                // 16-bit weights: widen, add, round into the format
        const bool bf = wt == 2u;
        const u64 n = D.n;
        const u64 base = (u64)(tile - D.tile_begin) * EXCP_TILE;
        const u32 rem = (n - base < (u64)EXCP_TILE) ? (u32)(n - base) : EXCP_TILE;
        if (t != cur_t) {
            __syncthreads();
            const EXCP_GLOBAL float *books = gptr((const float *)(D.blob + EXCP_HEADER));
            for (u32 i = tid; i < 3u * E; i += EXCP_THREADS) s_book[(i / E) * 256u + (i % E)] = books[i];
            cur_t = t;
            __syncthreads();
        }
        bool bad = false;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const u32 off = (u32)k * 2048u + tid * 8u;
            if (off >= rem) continue;
            const u32 left = min(8u, rem - off);
            const u64 e0 = base + off;
            const unsigned char *src[3] = {D.cw, D.cm, D.cv};
            float *dst[3] = {D.W_out, D.m_out, D.v_out};
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                if (dst[q] == nullptr) continue;
                // the eight codes, one byte each
                u64 c8 = 0;
                if (wide) {
                    const EXCP_GLOBAL unsigned char *p = gptr(src[q]) + e0;
                    if (left == 8u) c8 = *(const EXCP_GLOBAL u64 *)p;
                    else for (u32 j = 0; j < left; ++j) c8 |= (u64)p[j] << (8u * j);
                } else {
                    const EXCP_GLOBAL unsigned char *p = gptr(src[q]) + (e0 >> 1);
                    u32 c4 = 0;
                    if (left == 8u) c4 = *(const EXCP_GLOBAL u32 *)p;
                    else {
                        for (u32 j = 0; j < (left + 1u) / 2u; ++j) c4 |= (u32)p[j] << (8u * j);
                        if ((left & 1u) && (c4 >> (4u * left))) bad = true;      // the unused half of the last byte
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) c8 |= (u64)((c4 >> (4 * j)) & 15u) << (8 * j);
                }
                float x[8];
                EXCP_GLOBAL float *out = gptr(dst[q]) + e0;
                if (q == 0 && wt != 0u) {
                    const EXCP_GLOBAL unsigned short *Hp = gptr((const unsigned short *)D.Wp) + e0;
                    EXCP_GLOBAL unsigned short *Ho = gptr((unsigned short *)D.W_out) + e0;
                    u32 h[8];
                    const bool vec = left == 8u && (((uintptr_t)D.Wp | (uintptr_t)D.W_out) & 7u) == 0u;
                    if (vec) {
                        const us4 a = *(const EXCP_GLOBAL us4 *)Hp, b = *(const EXCP_GLOBAL us4 *)(Hp + 4);
#pragma unroll
                        for (int j = 0; j < 4; ++j) { h[j] = a[j]; h[4 + j] = b[j]; }
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) h[j] = ((u32)j < left) ? Hp[j] : 0u;
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const u32 c = (u32)(c8 >> (8 * j)) & 255u;
                        if (c >= E) bad = true;
                        const float centre = s_book[c & (E - 1u)];
                        if (c) h[j] = w16_narrow(w16_widen(h[j], bf) + centre, bf);
                    }
                    if (vec) {
                        us4 a, b;
#pragma unroll
                        for (int j = 0; j < 4; ++j) { a[j] = (unsigned short)h[j]; b[j] = (unsigned short)h[4 + j]; }
                        *(EXCP_GLOBAL us4 *)Ho = a; *(EXCP_GLOBAL us4 *)(Ho + 4) = b;
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) if ((u32)j < left) Ho[j] = (unsigned short)h[j];
                    }
                    continue;
                }
                if (q == 0) {
                    const EXCP_GLOBAL float *Wp = gptr(D.Wp) + e0;
                    if (left == 8u) {
                        const f4u a = *(const EXCP_GLOBAL f4u *)Wp, b = *(const EXCP_GLOBAL f4u *)(Wp + 4);
                        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) x[j] = ((u32)j < left) ? Wp[j] : 0.f;
                    }
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const u32 c = (u32)(c8 >> (8 * j)) & 255u;
                    if (c >= E) bad = true;
                    const float centre = s_book[(u32)q * 256u + (c & (E - 1u))];
                    if (q == 0) x[j] = c ? x[j] + centre : x[j];
                    else x[j] = c ? centre : 0.f;
                }
                if (left == 8u) {
                    f4u a, b;
                    a.x = x[0]; a.y = x[1]; a.z = x[2]; a.w = x[3]; b.x = x[4]; b.y = x[5]; b.z = x[6]; b.w = x[7];
                    *(EXCP_GLOBAL f4u *)out = a; *(EXCP_GLOBAL f4u *)(out + 4) = b;
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) if ((u32)j < left) out[j] = x[j];
                }
            }
        }
        if (bad) S.status = -40;
    }
}

// -40 (damage seen while decoding) becomes the public "damaged blob" status.
__global__ void k_dense_status(Workspace w, u32 ntensors) {
    const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < ntensors && w.dst[t].status == -40) w.dst[t].status = -4;
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
    D.cw = nullptr; D.cm = nullptr; D.cv = nullptr; D.head = nullptr; D.wtype = excp_wtype(g.flags); D.pad = 0;
    D.tile_begin = C.tile_begin; D.tile_count = C.tile_count;
    S.n_w = T.n_w; S.n_o = T.n_o; S.blob_bytes = T.blob_bytes; S.nbits = (u32)g.nbits;
    S.off_bw = EXCP_HEADER + excp_books_bytes((u32)g.nbits);
    S.off_bo = T.off_bo; S.off_cw = T.off_cw; S.off_cm = T.off_cm; S.off_cv = T.off_cv;
    S.status = (T.status == 0 && C.W_out != nullptr) ? 0 : 1;    // 1 = skip silently
    S.pop_w = 0; S.pop_o = 0; S.flags = g.flags; S.pad = 0;
    if (t == 0) *w.dec_kinds = blob_kind((u32)g.nbits, g.flags);
}

// The compress path already knows how many survivors precede every tile: the exclusive scan of its
// mask pass, taken at the tile's first sub-tile.
__global__ void k_decode_counts_from_mask(Workspace w, u32 ntiles) {
    const u32 tile = blockIdx.x * blockDim.x + threadIdx.x;
    if (tile < ntiles) w.dec_cnt_w[tile] = (u32)(w.mask_prefix[2ull * tile] >> 32);
}

// The descriptor of a single-tensor call arrives as a kernel argument and is written into the tables
// the decoders read (for callers that have no staging memory to copy it from).
__global__ void k_decode_single_setup(Workspace w, DDesc d) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        w.ddesc[0] = d;
        w.tile_begin[0] = 0u;
        w.tile_begin[1] = d.tile_count;
    }
}

}  // namespace

void launch_decode_single_setup(const Workspace &w, const DDesc &d, hipStream_t s) {
    hipLaunchKernelGGL(k_decode_single_setup, dim3(1), dim3(64), 0, s, w, d);
}

void launch_decode_parse(const Workspace &w, u32 ntensors, bool allow_raw, hipStream_t s) {
    if (!ntensors) return;
    launch_zero_u32(w.dec_kinds, 1, s);
    hipLaunchKernelGGL(k_decode_parse, dim3((ntensors + 255) / 256), dim3(256), 0, s, w, ntensors, allow_raw ? 1u : 0u);
}
void launch_decode_from_compress(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_decode_from_compress, dim3((g.ntensors + 255) / 256), dim3(256), 0, s, w, g);
    if (g.ntiles) hipLaunchKernelGGL(k_decode_counts_from_mask, dim3((g.ntiles + 255) / 256), dim3(256), 0, s, w, g.ntiles);
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
    const dim3 grid(ntensors * DSCAN_PARTS), block(EXCP_THREADS);
    if (which == 0) {
        hipLaunchKernelGGL(k_decode_scan_parts<0>, grid, block, 0, s, w, ntensors);
        hipLaunchKernelGGL(k_decode_scan<0>, grid, block, 0, s, w, ntensors);
    } else {
        hipLaunchKernelGGL(k_decode_scan_parts<1>, grid, block, 0, s, w, ntensors);
        hipLaunchKernelGGL(k_decode_scan<1>, grid, block, 0, s, w, ntensors);
    }
}
void launch_decode_main(const Workspace &w, u32 ntensors, u32 ntiles, bool moments, hipStream_t s) {
    if (!ntiles) return;
    u32 blocks = excp_grid(w, 64);
    if (blocks > ntiles) blocks = ntiles;
    if (moments) hipLaunchKernelGGL(k_decode_main<true>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
    else hipLaunchKernelGGL(k_decode_main<false>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
}
void launch_decode_main16(const Workspace &w, u32 ntensors, u32 ntiles, bool moments, hipStream_t s) {
    if (!ntiles) return;
    u32 blocks = excp_grid(w, 64);
    if (blocks > ntiles) blocks = ntiles;
    if (moments) hipLaunchKernelGGL(k_decode_main16<true>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
    else hipLaunchKernelGGL(k_decode_main16<false>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
}
void launch_decode_raw(const Workspace &w, u32 ntensors, u32 ntiles, bool moments, hipStream_t s) {
    if (!ntiles) return;
    u32 blocks = excp_grid(w, 32);
    if (blocks > ntiles) blocks = ntiles;
    if (moments) hipLaunchKernelGGL(k_decode_raw<true>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
    else hipLaunchKernelGGL(k_decode_raw<false>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
}
void launch_export_dense(const Workspace &w, u32 ntensors, u32 ntiles, bool moments, hipStream_t s) {
    if (!ntensors) return;
    hipLaunchKernelGGL(k_export_head, dim3(ntensors), dim3(EXCP_THREADS), 0, s, w, ntensors);
    if (!ntiles) return;
    u32 blocks = excp_grid(w, 64);
    if (blocks > ntiles) blocks = ntiles;
    if (moments) hipLaunchKernelGGL(k_export_dense<true>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
    else hipLaunchKernelGGL(k_export_dense<false>, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
}
void launch_dense_parse(const Workspace &w, u32 ntensors, hipStream_t s) {
    if (!ntensors) return;
    hipLaunchKernelGGL(k_dense_parse, dim3((ntensors + 255) / 256), dim3(256), 0, s, w, ntensors);
}
void launch_decode_dense(const Workspace &w, u32 ntensors, u32 ntiles, hipStream_t s) {
    if (!ntensors) return;
    if (ntiles) {
        u32 blocks = excp_grid(w, 32);
        if (blocks > ntiles) blocks = ntiles;
        hipLaunchKernelGGL(k_decode_dense, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
    }
    hipLaunchKernelGGL(k_dense_status, dim3((ntensors + 255) / 256), dim3(256), 0, s, w, ntensors);
}
void launch_decode_finish(const Workspace &w, u32 ntensors, hipStream_t s) {
    if (!ntensors) return;
    hipLaunchKernelGGL(k_decode_finish, dim3((ntensors + 255) / 256), dim3(256), 0, s, w, ntensors, w.rec_base);
}
void launch_decode_chain(const Workspace &w, u32 ntensors, u32 ntiles, hipStream_t s) {
    if (!ntiles) return;
    u32 blocks = excp_grid(w, 64);
    if (blocks > ntiles) blocks = ntiles;
    hipLaunchKernelGGL(k_decode_chain, dim3(blocks), dim3(EXCP_THREADS), 0, s, w, ntensors, ntiles);
}
void launch_chain_finish(const Workspace &w, u32 ntensors, hipStream_t s) {
    if (!ntensors) return;
    hipLaunchKernelGGL(k_chain_finish, dim3((ntensors + 255) / 256), dim3(256), 0, s, w, ntensors, w.rec_base);
}
