// Joint pruning masks (Sec. 3.2, Eq. "r_w" and Eq. "r_o") fused with an order-preserving stream
// compaction of the survivors, in one pass over W_prev, W_t, m and v.
//
// A tile is 4096 elements: 4 waves x 16 batches of 64, so that one wave ballot is one word of the
// keep bitmap.  Survivor positions need the number of survivors in all earlier tiles of the same
// tensor; tiles publish (aggregate, inclusive prefix) status words and look back over their
// predecessors (single-pass chained scan).  Workgroups are persistent and take tiles b, b+G, ...
// with every workgroup resident, so the tile a workgroup waits for is always owned by a running
// workgroup; a bounded spin turns any violation of that into an error flag instead of a hang.
#include "excp_util.h"

namespace {

__device__ __forceinline__ u64 pack_status(u32 flag, u32 cw, u32 co) {
    return ((u64)flag << 62) | ((u64)cw << 31) | (u64)co;
}

__global__ __launch_bounds__(EXCP_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_mask_compact(Workspace w, GroupParams g) {
    __shared__ u32 s_w[4], s_o[4], s_excl[2];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u64 lt_mask = lanemask_lt();

    for (u32 tile = blockIdx.x; tile < g.ntiles; tile += gridDim.x) {
        const u32 t = find_owner(w.tile_begin, g.ntensors, tile);
        const TDesc &D = w.desc[t];
        const u64 n = D.n;
        const u32 ltile = tile - D.tile_begin;
        const u64 base = (u64)ltile * EXCP_TILE;
        const float t_w = w.st[t].t_w, r_o = w.st[t].r_o;
        const float *__restrict__ Wp = D.Wp, *__restrict__ W = D.W, *__restrict__ M = D.m, *__restrict__ V = D.v;

        float dv[16], mv[16], vv[16];
        u64 bw[16], bo[16];
        u32 nf = 0, cw = 0, co = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            u64 idx = base + (u64)((wave * 16 + j) * 64 + lane);
            bool ok = idx < n;
            float a = ok ? W[idx] : 0.f;
            float p = ok ? Wp[idx] : 0.f;
            mv[j] = ok ? M[idx] : 0.f;
            vv[j] = ok ? V[idx] : 1.f;
            dv[j] = a - p;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            u64 idx = base + (u64)((wave * 16 + j) * 64 + lane);
            bool ok = idx < n;
            float r = __fdiv_rn(t_w, __fsqrt_rn(vv[j]));
            bool kw = ok && (fabsf(dv[j]) > r);
            bool ko = kw && (fabsf(mv[j]) > r_o);
            nf += ((f2u(vv[j]) & 0x7f800000u) == 0x7f800000u);
            bw[j] = ballot64(kw);
            bo[j] = ballot64(ko);
            cw += __popcll(bw[j]);
            co += __popcll(bo[j]);
        }
        // keep bitmap of the residual: one ballot per 64 elements
        {
            u64 *bm = (u64 *)(D.blob + EXCP_HEADER + 12ull * (1u << g.nbits));
            const u64 nwords = excp_words(n);
            u64 mine = 0;
#pragma unroll
            for (int j = 0; j < 16; ++j) if (lane == (u32)j) mine = bw[j];
            u64 word = (base >> 6) + wave * 16 + lane;
            // words past the last element carry an all-zero ballot: that is the 16-byte padding
            if (lane < 16 && word < nwords + (nwords & 1ull)) bm[word] = mine;
        }
        nf = wave_sum_u32(nf);
        if (lane == 0) {
            s_w[wave] = cw; s_o[wave] = co;
            if (nf) atomicAdd(&w.st[t].nonfinite, (u64)nf);
        }
        __syncthreads();
        const u32 tw = s_w[0] + s_w[1] + s_w[2] + s_w[3];
        const u32 to = s_o[0] + s_o[1] + s_o[2] + s_o[3];

        if (wave == 0) {
            u32 ew = 0, eo = 0;
            u64 *status = w.tile_status;
            if (ltile != 0) {
                if (lane == 0) st_status(&status[tile], pack_status(1, tw, to));
                long long pos = (long long)tile - 1;
                const long long first = (long long)D.tile_begin;
                u32 spins = 0;
                bool giveup = false;
                u64 total = 0;                                   // packed: survivors << 31 | moment survivors
                while (true) {
                    // 256 predecessors per step: lane l reads tiles pos - l, pos - 64 - l, ...
                    u64 sv[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        long long idx = pos - (long long)(q * 64 + lane);
                        sv[q] = (idx >= first) ? ld_status(&status[idx]) : pack_status(2, 0, 0);
                    }
                    u64 part = 0;
                    bool done = false, retry = false;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (done || retry) continue;
                        const u32 flag = (u32)(sv[q] >> 62);
                        const u64 m2 = ballot64(flag == 2u);
                        const u64 m0 = ballot64(flag == 0u);
                        u64 want = ~0ull;
                        if (m2) { int L = __ffsll((long long)m2) - 1; want = (L == 63) ? ~0ull : ((1ull << (L + 1)) - 1ull); }
                        if (m0 & want) { retry = true; continue; }
                        if ((want >> lane) & 1ull) part += sv[q] & 0x3fffffffffffffffull;
                        if (m2) done = true;
                    }
                    if (retry) {
                        if (++spins > EXCP_SPIN_LIMIT) { giveup = true; break; }
                        __builtin_amdgcn_s_sleep(1);
                        continue;
                    }
                    total += wave_sum_u64(part);
                    if (done) break;
                    pos -= 256;
                }
                ew = (u32)(total >> 31);
                eo = (u32)(total & 0x7fffffffull);
                if (giveup && lane == 0) atomicExch(w.err_flag, 1);
            }
            if (lane == 0) {
                st_status(&status[tile], pack_status(2, ew + tw, eo + to));
                s_excl[0] = ew; s_excl[1] = eo;
                if (base + EXCP_TILE >= n) { w.st[t].n_w = (u64)ew + tw; w.st[t].n_o = (u64)eo + to; }
            }
        }
        __syncthreads();
        u32 pw = s_excl[0], po = s_excl[1];
        for (u32 q = 0; q < wave; ++q) { pw += s_w[q]; po += s_o[q]; }

        float *__restrict__ xw = w.xw + D.elem_off;
        float *__restrict__ xm = w.xm + D.elem_off;
        float *__restrict__ xv = w.xv + D.elem_off;
        // M_o restricted to the survivors, as a bit stream that starts at survivor position pw
        const u64 off_bo = EXCP_HEADER + 12ull * (1u << g.nbits) + excp_pad16(8ull * excp_words(n));
        u64 *bmo = (u64 *)(D.blob + off_bo);
        const u64 cap_words = (D.blob_cap > off_bo) ? (D.blob_cap - off_bo) >> 3 : 0ull;
        u64 acc = 0;
        u32 fill = pw & 63u;
        u64 wordidx = pw >> 6;
        bool first = true;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const u64 mw = bw[j], mo = bo[j];
            const bool kw = (mw >> lane) & 1ull, ko = (mo >> lane) & 1ull;
            const u32 nb = __popcll(mw);
            const u32 rk = __popcll(mw & lt_mask);
            const u32 ro = __popcll(mo & lt_mask);
            if (kw) xw[pw + rk] = dv[j];
            if (ko) { xm[po + ro] = mv[j]; xv[po + ro] = vv[j]; }
            // move each survivor's M_o bit to lane = its rank among the survivors of this batch
            const u32 dest = kw ? rk : nb + (lane - rk);
            const int got = __builtin_amdgcn_ds_permute((int)(dest << 2), ko ? 1 : 0);
            const u64 cbits = ballot64(got != 0);
            if (nb) {
                acc |= cbits << fill;
                if (fill + nb >= 64u) {
                    if (lane == 0 && wordidx < cap_words) {
                        if (first) atomicOr(&bmo[wordidx], acc); else bmo[wordidx] = acc;
                    }
                    first = false;
                    acc = fill ? (cbits >> (64u - fill)) : 0ull;
                    ++wordidx;
                    fill = fill + nb - 64u;
                } else {
                    fill += nb;
                }
            }
            pw += nb;
            po += __popcll(mo);
        }
        if (fill && lane == 0 && wordidx < cap_words && acc) atomicOr(&bmo[wordidx], acc);
        __syncthreads();
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
            u64 off = EXCP_HEADER + 12ull * (1u << g.nbits) + excp_pad16(8ull * excp_words(n));
            S.off_bo = off; off += excp_pad16(8ull * excp_words(nw));
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
            u64 off = EXCP_HEADER + 12ull * (1u << g.nbits) + excp_pad16(8ull * excp_words(n));
            off += excp_pad16(8ull * excp_words(nw)) + excp_pad16(8ull * excp_words(nw * nb)) +
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

int query_persistent_grid(int device) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return -1;
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k_mask_compact, EXCP_THREADS, 0) != hipSuccess || nb <= 0)
        return -1;
    return nb * prop.multiProcessorCount;
}

void launch_mask_compact(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntiles) return;
    hipLaunchKernelGGL(k_mask_compact, dim3(w.grid_persistent), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_layout(const Workspace &w, const GroupParams &g, hipStream_t s) {
    hipLaunchKernelGGL(k_layout, dim3(1), dim3(EXCP_THREADS), 0, s, w, g, w.seg_chunk_begin);
}
