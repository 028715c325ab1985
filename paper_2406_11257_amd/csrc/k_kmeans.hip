// Non-uniform quantisation of the surviving values (Sec. 3.3): per stream, K = 2^nbits - 1
// centres by Lloyd's algorithm, then codes = 1 + nearest centre packed nbits each (Sec. 4.2).
//
//   init      : the K order statistics of rank ((2k+1) len)/(2K), found exactly by a three-pass
//               multi-rank radix select over order-preserving 32-bit keys (12 + 10 + 10 bits);
//   iteration : every workgroup keeps the centres in LDS, accumulates per-centre (fp64 sum, count)
//               for its chunk in lane-private LDS bins, reduces them in a fixed order and writes one
//               partial per chunk; a second kernel adds the partials in chunk order and moves the
//               centres.  Nothing is accumulated with floating-point atomics when K <= 15, so the
//               result does not depend on scheduling;
//   final     : nearest final centre, objective, bit packing into the blob's code sections.
//
// All survivor passes walk one chunk list (8192 values per chunk) that spans every stream of every
// tensor of the group; its length is only known on the device.
#include "excp_util.h"

namespace {

__device__ __forceinline__ const float *seg_data(const Workspace &w, u32 sidx) {
    const u32 t = sidx / 3u, which = sidx % 3u;
    const float *basep = which == 0 ? w.xw : (which == 1 ? w.xm : w.xv);
    return basep + w.desc[t].elem_off;
}

// ------------------------------------------------------------------ multi-rank select, histograms
// PASS 1: 4096-bin histogram of key >> 20 per stream (LDS, flushed when the stream changes).
// PASS 2: for keys whose top 12 bits are a live prefix: 1024-bin histogram of bits 19..10 per slot.
// PASS 3: for keys whose top 22 bits are a live prefix: 1024-bin histogram of bits 9..0 per slot.
template <int PASS, bool LDS_SLOTS>
__global__ __launch_bounds__(EXCP_THREADS) void k_init_hist(Workspace w, GroupParams g) {
    extern __shared__ u32 smem[];
    // PASS 1: smem = hist[4096]
    // PASS 2: smem = bin2slot bytes [4096] (as 1024 u32) followed by hist[slots][1024] when LDS_SLOTS
    // PASS 3: smem = slot_prefix[256]
    const u32 tid = threadIdx.x;
    const u32 total = *w.chunk_total;
    const u32 G = gridDim.x, b = blockIdx.x;
    const u32 lo = (u32)(((u64)b * total) / G), hi = (u32)(((u64)(b + 1) * total) / G);
    if (lo >= hi) return;
    const u32 nseg = 3u * g.ntensors;
    const u32 K = (u32)g.K;
    const u32 lds_slots = K < 15u ? K : 15u;

    u32 sidx = find_owner(w.seg_chunk_begin, nseg, lo);
    u32 s_end = w.seg_chunk_begin[sidx + 1];

    auto enter = [&](u32 sg) {
        if (PASS == 1) {
            for (u32 i = tid; i < 4096u; i += EXCP_THREADS) smem[i] = 0;
        } else if (PASS == 2) {
            const u32 *src = w.bin2slot + (u64)sg * 1024u;
            for (u32 i = tid; i < 1024u; i += EXCP_THREADS) smem[i] = src[i];
            if (LDS_SLOTS) for (u32 i = tid; i < lds_slots * 1024u; i += EXCP_THREADS) smem[1024u + i] = 0;
        } else {
            const SegState &S = w.seg[sg];
            for (u32 i = tid; i < 256u; i += EXCP_THREADS) smem[i] = (i < S.nslots) ? S.slot_prefix[i] : 0xffffffffu;
        }
        __syncthreads();
    };
    auto leave = [&](u32 sg) {
        __syncthreads();
        if (PASS == 1) {
            u32 *dst = w.hist1 + (u64)sg * 4096u;
            for (u32 i = tid; i < 4096u; i += EXCP_THREADS) { u32 c = smem[i]; if (c) atomicAdd(&dst[i], c); }
        } else if (PASS == 2 && LDS_SLOTS) {
            u32 *dst = w.hist2 + (u64)sg * w.hist2_slots * 1024u;
            const u32 ns = w.seg[sg].nslots;
            for (u32 i = tid; i < ns * 1024u; i += EXCP_THREADS) { u32 c = smem[1024u + i]; if (c) atomicAdd(&dst[i], c); }
        }
        __syncthreads();
    };

    enter(sidx);
    for (u32 c = lo; c < hi; ++c) {
        if (c >= s_end) {
            leave(sidx);
            sidx = find_owner(w.seg_chunk_begin, nseg, c);
            s_end = w.seg_chunk_begin[sidx + 1];
            enter(sidx);
        }
        const SegState &S = w.seg[sidx];
        const float *__restrict__ x = seg_data(w, sidx);
        const u64 len = S.len;
        const u64 base = (u64)(c - S.chunk_begin) * EXCP_CHUNK;
        const u32 nslots = S.nslots;
        u32 *gh = w.hist2 + (u64)sidx * w.hist2_slots * 1024u;
        const unsigned char *b2s = (const unsigned char *)smem;
#pragma unroll 4
        for (u32 it = 0; it < EXCP_CHUNK / EXCP_THREADS; ++it) {
            u64 idx = base + (u64)it * EXCP_THREADS + tid;
            if (idx < len) {
                u32 k = key_of(x[idx]);
                if (PASS == 1) {
                    atomicAdd(&smem[k >> 20], 1u);
                } else if (PASS == 2) {
                    u32 slot = b2s[k >> 20];
                    if (slot != 0xffu) {
                        u32 bin = (k >> 10) & 1023u;
                        if (LDS_SLOTS) atomicAdd(&smem[1024u + slot * 1024u + bin], 1u);
                        else atomicAdd(&gh[(u64)slot * 1024u + bin], 1u);
                    }
                } else {
                    u32 p = k >> 10;
                    u32 l = 0, h = nslots;            // lower bound of p among the sorted live prefixes
                    while (l < h) { u32 mid = (l + h) >> 1; if (smem[mid] < p) l = mid + 1; else h = mid; }
                    if (l < nslots && smem[l] == p) atomicAdd(&gh[(u64)l * 1024u + (k & 1023u)], 1u);
                }
            }
        }
    }
    leave(sidx);
}

// ------------------------------------------------------------------ multi-rank select, resolve
// One workgroup per stream.  After pass 1 the wanted ranks are placed in the 4096-bin histogram;
// after passes 2 and 3 each rank descends inside the 1024-bin histogram of its slot.  Live prefixes
// are kept sorted and distinct ("slots").
template <int PASS>
__global__ __launch_bounds__(EXCP_THREADS) void k_init_resolve(Workspace w, GroupParams g) {
    __shared__ u32 s_sum[EXCP_THREADS];
    __shared__ u32 s_prefix[EXCP_MAX_K + 1];
    const u32 sidx = blockIdx.x, tid = threadIdx.x;
    SegState &S = w.seg[sidx];
    const u64 len = S.len;
    const u32 K = (u32)g.K;
    if (len == 0) {
        if (PASS == 3) for (u32 k = tid; k < K; k += EXCP_THREADS) S.C[k] = 0.f;
        if (PASS == 1 && tid == 0) S.nslots = 0;
        return;
    }
    if (PASS == 1) {
        u32 *H = w.hist1 + (u64)sidx * 4096u;
        u32 c[16], local = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) { c[i] = H[tid * 16 + i]; local += c[i]; H[tid * 16 + i] = 0; }
        s_sum[tid] = local;
        __syncthreads();
        for (int off = 1; off < EXCP_THREADS; off <<= 1) {
            u32 v = (tid >= (u32)off) ? s_sum[tid - off] : 0u;
            __syncthreads();
            s_sum[tid] += v;
            __syncthreads();
        }
        // every rank k finds the thread whose bins contain it
        for (u32 k = 0; k < K; ++k) {
            u32 r = (u32)(((u64)(2 * k + 1) * len) / (2ull * K));
            u32 before = s_sum[tid] - local;
            if (r >= before && r < before + local) {
                u32 rr = r - before;
                int i = 0;
                while (rr >= c[i]) { rr -= c[i]; ++i; }
                S.prefix[k] = tid * 16 + i;
                S.rank[k] = rr;
                s_prefix[k] = tid * 16 + i;
            }
        }
    } else {
        const u32 *H = w.hist2 + (u64)sidx * w.hist2_slots * 1024u;
        for (u32 k = tid; k < K; k += EXCP_THREADS) {
            const u32 *h = H + (u64)S.slot_of_rank[k] * 1024u;
            u32 r = S.rank[k], bin = 0;
            while (bin < 1023u) { u32 cnt = h[bin]; if (r < cnt) break; r -= cnt; ++bin; }
            u32 np = (S.prefix[k] << 10) | bin;
            S.prefix[k] = np;
            S.rank[k] = r;
            s_prefix[k] = np;
            if (PASS == 3) S.C[k] = val_of(np);
        }
    }
    __syncthreads();
    if (PASS != 3 && tid == 0) {
        // ranks ascend, so prefixes are non-decreasing: distinct ones in order are the slots
        u32 ns = 0;
        for (u32 k = 0; k < K; ++k) {
            if (k == 0 || s_prefix[k] != s_prefix[k - 1]) { S.slot_prefix[ns] = s_prefix[k]; ++ns; }
            S.slot_of_rank[k] = ns - 1;
        }
        S.nslots = ns;
    }
    __syncthreads();
    if (PASS == 1) {
        // byte table: top-12-bit bin -> slot (0xff = not wanted)
        u32 *tab = w.bin2slot + (u64)sidx * 1024u;
        const u32 ns = S.nslots;
        for (u32 i = tid; i < 1024u; i += EXCP_THREADS) {
            u32 packed = 0;
            for (u32 q = 0; q < 4; ++q) {
                u32 bin = i * 4 + q, slot = 0xffu;
                u32 l = 0, h = ns;
                while (l < h) { u32 mid = (l + h) >> 1; if (S.slot_prefix[mid] < bin) l = mid + 1; else h = mid; }
                if (l < ns && S.slot_prefix[l] == bin) slot = l;
                packed |= slot << (8 * q);
            }
            tab[i] = packed;
        }
    }
    if (PASS == 2 || PASS == 3) {
        // clear the slot histograms this stream used (ready for the next pass / next batch)
        u32 *H = w.hist2 + (u64)sidx * w.hist2_slots * 1024u;
        const u32 used = (PASS == 2) ? w.seg[sidx].nslots : K;   // upper bound of slots written
        u32 lim = used > w.hist2_slots ? (u32)w.hist2_slots : used;
        for (u32 i = tid; i < lim * 1024u; i += EXCP_THREADS) H[i] = 0;
    }
}

// ------------------------------------------------------------------ Lloyd accumulation
// K <= 15: bins are private to a lane ([k][tid] layout, conflict free).  K > 15: bins are shared by
// the workgroup and filled with LDS atomics.
template <bool SMALLK>
__global__ __launch_bounds__(EXCP_THREADS) void k_lloyd_accum(Workspace w, GroupParams g) {
    extern __shared__ unsigned char smraw[];
    __shared__ float s_C[EXCP_MAX_K + 1];
    const u32 tid = threadIdx.x, lane = tid & 63u;
    const u32 total = *w.chunk_total;
    const u32 G = gridDim.x, b = blockIdx.x;
    const u32 lo = (u32)(((u64)b * total) / G), hi = (u32)(((u64)(b + 1) * total) / G);
    if (lo >= hi) return;
    const u32 nseg = 3u * g.ntensors;
    const int K = g.K;
    double *bsum = (double *)smraw;                                   // SMALLK: [16][256]; else [256]
    u32 *bcnt = (u32 *)(smraw + (SMALLK ? 16 * EXCP_THREADS * 8 : 256 * 8));

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
        const float *__restrict__ x = seg_data(w, sidx);
        const u64 len = S.len;
        const u64 base = (u64)(c - S.chunk_begin) * EXCP_CHUNK;
        if (SMALLK) {
#pragma unroll
            for (int k = 0; k < 16; ++k) { bsum[k * EXCP_THREADS + tid] = 0.0; bcnt[k * EXCP_THREADS + tid] = 0; }
        } else {
            if (tid < 256) { bsum[tid] = 0.0; bcnt[tid] = 0; }
            __syncthreads();
        }
#pragma unroll 4
        for (u32 it = 0; it < EXCP_CHUNK / EXCP_THREADS; ++it) {
            u64 idx = base + (u64)it * EXCP_THREADS + tid;
            if (idx < len) {
                float xv = x[idx];
                int a = nearest_centre(xv, s_C, K, nullptr);
                if (SMALLK) {
                    bsum[a * EXCP_THREADS + tid] += (double)xv;
                    bcnt[a * EXCP_THREADS + tid] += 1u;
                } else {
                    atomicAdd(&bsum[a], (double)xv);
                    atomicAdd(&bcnt[a], 1u);
                }
            }
        }
        __syncthreads();
        double *ps = w.part_sum + (u64)c * (u32)K;
        u32 *pc = w.part_cnt + (u64)c * (u32)K;
        if (SMALLK) {
            // thread (k = tid / 16, part = tid % 16) adds 16 lane bins in order, then a 16-lane tree
            const u32 k = tid >> 4, part = tid & 15u;
            double sacc = 0.0; u32 cacc = 0;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                sacc += bsum[k * EXCP_THREADS + part * 16 + q];
                cacc += bcnt[k * EXCP_THREADS + part * 16 + q];
            }
#pragma unroll
            for (int mm = 8; mm >= 1; mm >>= 1) {
                sacc += shfl_xor_f64(sacc, mm);
                cacc += __shfl_xor(cacc, mm, WAVE);
            }
            if (part == 0 && k < (u32)K) { ps[k] = sacc; pc[k] = cacc; }
            (void)lane;
        } else {
            for (u32 k = tid; k < (u32)K; k += EXCP_THREADS) { ps[k] = bsum[k]; pc[k] = bcnt[k]; }
        }
        __syncthreads();
    }
}

// One workgroup per stream: add the chunk partials in a fixed order and move the centres.
__global__ __launch_bounds__(EXCP_THREADS) void k_lloyd_update(Workspace w, GroupParams g) {
    const u32 sidx = blockIdx.x, tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    SegState &S = w.seg[sidx];
    if (S.len == 0) return;
    const u32 K = (u32)g.K;
    const u32 c0 = S.chunk_begin, c1 = w.seg_chunk_begin[sidx + 1];
    for (u32 k = wave; k < K; k += 4) {
        double sacc = 0.0; u64 cacc = 0;
        for (u32 c = c0 + lane; c < c1; c += 64) {
            sacc += w.part_sum[(u64)c * K + k];
            cacc += w.part_cnt[(u64)c * K + k];
        }
#pragma unroll
        for (int mm = 32; mm >= 1; mm >>= 1) {
            sacc += shfl_xor_f64(sacc, mm);
            cacc += shfl_xor_u64(cacc, mm);
        }
        if (lane == 0 && cacc) S.C[k] = (float)(sacc / (double)cacc);
    }
}

// ------------------------------------------------------------------ final assignment + packing
__global__ __launch_bounds__(EXCP_THREADS) void k_assign_pack(Workspace w, GroupParams g) {
    __shared__ float s_C[EXCP_MAX_K + 1];
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
        const u64 nwords = excp_words(len * nbits);
        u64 *out = (u64 *)(w.desc[t].blob + (which == 0 ? T.off_cw : (which == 1 ? T.off_cm : T.off_cv)));
        const u64 wbase = (u64)(c - S.chunk_begin) * words_per_chunk;
        double obj = 0.0;
        for (u32 wl = tid; wl < words_per_chunk; wl += EXCP_THREADS) {
            const u64 wg = wbase + wl;
            if (wg >= nwords) break;
            const u64 bit0 = wg * 64ull;
            u64 e = bit0 / nbits;
            u64 word = 0;
            while (e < len && e * nbits < bit0 + 64ull) {
                double dist;
                const u32 code = 1u + (u32)nearest_centre(x[e], s_C, K, &dist);
                const long long sh = (long long)(e * nbits) - (long long)bit0;
                if (sh >= 0) { word |= (u64)code << sh; obj += dist; }
                else word |= (u64)code >> (-sh);
                ++e;
            }
            out[wg] = word;
            if (wg == nwords - 1 && (nwords & 1ull)) out[nwords] = 0ull;     // 16-byte padding
        }
#pragma unroll
        for (int mm = 32; mm >= 1; mm >>= 1) obj += shfl_xor_f64(obj, mm);
        if (lane == 0) s_red[wave] = obj;
        __syncthreads();
        if (tid == 0) w.part_obj[c] = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
        (void)ebase;
        __syncthreads();
    }
}

// ------------------------------------------------------------------ header, codebooks, results
__global__ __launch_bounds__(EXCP_THREADS) void k_finalize(Workspace w, GroupParams g, u32 rec_base) {
    __shared__ double s_obj[3];
    const u32 t = blockIdx.x, tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const TDesc &D = w.desc[t];
    TState &T = w.st[t];
    const u32 E = 1u << g.nbits, K = (u32)g.K;
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
        // padding word of bitmap_o (the bitmap region was cleared before the masks were written)
        HostRec &R = w.rec_dev[rec_base + t];
        R.n = D.n; R.n_w = T.n_w; R.n_o = T.n_o; R.blob_bytes = T.blob_bytes; R.nonfinite = T.nonfinite;
        R.abs_sum = T.abs_sum; R.obj[0] = s_obj[0]; R.obj[1] = s_obj[1]; R.obj[2] = s_obj[2];
        R.med = u2f(T.med_bits); R.mean32 = T.mean32; R.t_w = T.t_w; R.r_o = T.r_o;
        R.status = status; R.pad = 0;
    }
    (void)K;
}

}  // namespace

static size_t init_hist_smem(int pass, bool lds_slots, int K) {
    if (pass == 1) return 4096 * 4;
    if (pass == 2) return 1024 * 4 + (lds_slots ? (size_t)(K < 15 ? K : 15) * 1024 * 4 : 0);
    return 256 * 4;
}

void launch_init_hist(const Workspace &w, const GroupParams &g, int pass, hipStream_t s) {
    dim3 grid(w.grid_stream), block(EXCP_THREADS);
    const bool lds = g.K <= 15;
    size_t sm = init_hist_smem(pass, lds, g.K);
    if (pass == 1) hipLaunchKernelGGL((k_init_hist<1, true>), grid, block, sm, s, w, g);
    else if (pass == 2 && lds) hipLaunchKernelGGL((k_init_hist<2, true>), grid, block, sm, s, w, g);
    else if (pass == 2) hipLaunchKernelGGL((k_init_hist<2, false>), grid, block, sm, s, w, g);
    else hipLaunchKernelGGL((k_init_hist<3, false>), grid, block, sm, s, w, g);
}

void launch_init_resolve(const Workspace &w, const GroupParams &g, int pass, hipStream_t s) {
    if (!g.ntensors) return;
    dim3 grid(3 * g.ntensors), block(EXCP_THREADS);
    if (pass == 1) hipLaunchKernelGGL(k_init_resolve<1>, grid, block, 0, s, w, g);
    else if (pass == 2) hipLaunchKernelGGL(k_init_resolve<2>, grid, block, 0, s, w, g);
    else hipLaunchKernelGGL(k_init_resolve<3>, grid, block, 0, s, w, g);
}

void launch_lloyd_accum(const Workspace &w, const GroupParams &g, hipStream_t s) {
    dim3 grid(w.grid_stream), block(EXCP_THREADS);
    if (g.K <= 15) hipLaunchKernelGGL(k_lloyd_accum<true>, grid, block, 16 * EXCP_THREADS * 12, s, w, g);
    else hipLaunchKernelGGL(k_lloyd_accum<false>, grid, block, 256 * 12, s, w, g);
}

void launch_lloyd_update(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_lloyd_update, dim3(3 * g.ntensors), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_assign_pack(const Workspace &w, const GroupParams &g, hipStream_t s) {
    hipLaunchKernelGGL(k_assign_pack, dim3(w.grid_stream), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_finalize(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_finalize, dim3(g.ntensors), dim3(EXCP_THREADS), 0, s, w, g, w.rec_base);
}
