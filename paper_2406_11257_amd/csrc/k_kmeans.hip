// Non-uniform quantisation of the surviving values (Sec. 3.3): per stream, K = 2^nbits - 1
// centres by Lloyd's algorithm, then codes = 1 + nearest centre packed nbits each (Sec. 4.2).
//
// One-dimensional Lloyd has structure that makes re-reading every value in every iteration
// unnecessary: clusters are intervals, and the assignment is monotone in the value.  So each stream
// is first PARTITIONED into 256 value-ordered buckets of roughly equal population, and for every
// bucket the exact count, exact sum, minimum and maximum are stored.  The bucket of a value comes
// from arithmetic and one table look-up: the magnitude's bit pattern, offset and shifted, names one
// of 2048 cells per sign (bit patterns of floats are ordered like the values, roughly
// logarithmically), and a sample of the stream decides which run of cells forms which bucket.
// In an iteration a bucket whose minimum and maximum go to the same centre contributes its stored
// totals; only the (at most K-1) buckets that a cluster border cuts are read element by element.
// The same buckets give the initial centres (order statistics of rank ((2k+1) len)/(2K)) with a
// radix select inside one bucket per rank.
//
// All sums are exact: a value is mant * 2^(pos-149); values that are neighbours in magnitude (inside
// a window of 24 binary orders) are whole multiples of one unit, small enough that sixteen of them add
// exactly in fp64; those partial sums go on as integers and end in signed 64-bit bins 8 binary orders
// apart (the representation of the exact sum of |m| in the statistics pass, here with sign); a value
// outside the window is filed into the bins by itself.  A centre is therefore
// fp32(round-once-fp64(exact sum) / count), independent of the order in which values were met, so
// integer atomics may be used freely and the partition need not be stable.
//
// The survivor passes walk one chunk list (8192 values per chunk) spanning every stream of every
// tensor of the group; its length is known only on the device.
#include "excp_util.h"

namespace {

constexpr u32 NBKT = 256;
constexpr u32 SAMPLE = 8192;
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

// Four consecutive floats at an address that is only known to be 4-byte aligned.
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

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

// Adds v * 2^(bitpos - 149) to a set of signed bins (bin g has weight 2^(8g - 149)), with integer atomics.
__device__ __forceinline__ void file_i64(u64 *bins, long long v, u32 bitpos) {
    const bool neg = v < 0;
    const u64 mag = neg ? (u64)0 - (u64)v : (u64)v;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const u64 piece = (mag >> (32 * q)) & 0xffffffffull;
        const u32 p = bitpos + 32u * q;
        const u64 d = piece << (p & 7u);
        if (piece) atomicAdd(&bins[p >> 3], neg ? (u64)0 - d : d);
    }
}

// Exact summation of values that are neighbours in magnitude.  A value inside the window of 24 bit
// positions [B, B + 24) is a whole multiple of the unit 2^(B-149) below 2^47 units, so up to sixteen of
// them add exactly in fp64, whatever their signs; such a partial sum is then split into two integers
// -- units below 2^32, and signed multiples of 2^32 units -- that go on in 64-bit integer counters.
struct WindowSum {
    double part = 0.0;             // at most sixteen values since the last fold
    long long lo = 0, hi = 0;      // sum = (lo + 2^32 hi) units
    __device__ __forceinline__ void fold(u32 B) {
        const double units = ldexp(part, 149 - (int)B);                  // an integer, |units| < 2^51
        const double h = floor(units * 2.3283064365386963e-10);          // floor(units / 2^32), |h| < 2^19
        lo += (long long)(u32)(units - h * 4294967296.0);
        hi += (long long)(int)h;
        part = 0.0;
    }
};
// magnitudes (bit patterns without the sign) inside the window: lo <= pattern < lo + span
__device__ __forceinline__ void window_range(u32 B, u32 &lo, u32 &span) {
    lo = B ? ((B + 1u) << 23) : 0u;
    span = ((B + 25u) << 23) - lo;
}

// Signed bins -> the exact sum rounded once (to nearest, ties to even) to fp64.
// Everything stays in registers (fixed indices after unrolling): this runs once per centre and
// iteration on the critical path between two small kernels.
__device__ double signed_bins_to_double(const u64 *bins) {
    // base-256 digits of the sum (bin g has weight 2^(8g)), what is left over in a signed top word
    u64 W[6] = {0, 0, 0, 0, 0, 0};
    long long carry = 0;
#pragma unroll
    for (int g = 0; g < EXCP_ABSM_BINS; ++g) {
        const u64 b = bins[g];
        const long long t = (long long)(b & 255ull) + carry;       // |carry| < 2^57: no overflow
        carry = (t >> 8) + ((long long)b >> 8);
        W[g >> 3] |= (u64)(t & 255) << (8 * (g & 7));
    }
    W[5] = (u64)carry;
    const bool neg = carry < 0;
    if (neg) {                                  // magnitude = two's complement negation of the 384 bits
        u64 c = 1;
#pragma unroll
        for (int i = 0; i < 6; ++i) { const u64 v = ~W[i] + c; c = (c && v == 0) ? 1ull : 0ull; W[i] = v; }
    }
    // the top non-zero word, the word below it, and whether anything lies below those
    u64 hi = 0, lo = 0, rest = 0; int wi = -1;
#pragma unroll
    for (int i = 5; i >= 0; --i) {
        if (wi < 0) { if (W[i]) { wi = i; hi = W[i]; } }
        else if (wi == i + 1) lo = W[i];
        else rest |= W[i];
    }
    if (wi < 0) return 0.0;
    const int top = 63 - __clzll((long long)hi), msb = 64 * wi + top;
    double mag;
    if (msb <= 52) {
        mag = ldexp((double)hi, -149);          // wi == 0: the value itself, exactly
    } else {
        // the 53 bits from msb down, out of hi:lo; sh = number of bits of hi:lo below them
        const int sh = top + 12;                // 64 + top - 52, in [12, 75]
        u64 mant, guard, sticky;
        if (sh < 64) {
            mant = (hi << (64 - sh)) | (lo >> sh);
            guard = (lo >> (sh - 1)) & 1ull;
            sticky = lo & ((1ull << (sh - 1)) - 1ull);
        } else if (sh == 64) {
            mant = hi; guard = lo >> 63; sticky = lo & 0x7fffffffffffffffull;
        } else {
            mant = hi >> (sh - 64);
            guard = (hi >> (sh - 65)) & 1ull;
            sticky = (hi & ((1ull << (sh - 65)) - 1ull)) | lo;
        }
        sticky |= rest;
        if (guard && (sticky || (mant & 1ull))) mant += 1;
        mag = ldexp((double)mant, msb - 52 - 149);
    }
    return neg ? -mag : mag;
}

// ---------------------------------------------------------------- P0: value -> bucket map from a sample
// One workgroup per stream.  The sample fixes the magnitude range of each sign (hence offset and
// shift of the cells); the cells' sample counts, scanned, give every cell its bucket so that the
// buckets hold about equal shares of the sample.
__global__ __launch_bounds__(EXCP_THREADS) void k_km_sample(Workspace w, GroupParams g) {
    __shared__ float smp[SAMPLE];
    __shared__ u32 cnt[EXCP_KM_CELLS];
    __shared__ u32 s_map[4];
    __shared__ u32 s_ext[4];                       // min / max magnitude of the negative, of the positive samples
    __shared__ u32 s_part[EXCP_THREADS];
    const u32 sidx = blockIdx.x, tid = threadIdx.x;
    const u64 len = w.seg[sidx].len;
    if (len == 0) return;
    // The stream is read where the mask pass left it, in the sub-tile slots (the dense copy is made
    // afterwards, by the pass that also counts the buckets this map defines): survivor p of the stream
    // sits in the sub-tile whose scanned count is the last one <= p.  Eight searches go side by side.
    const u32 ts = sidx / 3u, which = sidx % 3u;
    const u32 sub_first = 2u * w.tile_begin[ts], sub_end = 2u * w.tile_begin[ts + 1u];
    const u64 *pre = w.mask_prefix;
    const float *__restrict__ slots = (which == 0 ? w.pw : (which == 1 ? w.pm : w.pv)) + w.desc[ts].elem_off;
    const u32 ns = len < SAMPLE ? (u32)len : SAMPLE;
    if (tid < 4) s_ext[tid] = (tid & 1u) ? 0u : 0xffffffffu;
    for (u32 c = tid; c < EXCP_KM_CELLS; c += EXCP_THREADS) cnt[c] = 0;
    __syncthreads();
    u32 mn[2] = {0xffffffffu, 0xffffffffu}, mx[2] = {0u, 0u};
    for (u32 i0 = tid; i0 < ns; i0 += 8u * EXCP_THREADS) {
        u32 pos[8], lo[8], hi[8];
#pragma unroll
        for (u32 k = 0; k < 8; ++k) {
            const u32 i = min(i0 + k * EXCP_THREADS, ns - 1u);
            pos[k] = (u32)(((u64)i * len) / ns);
            lo[k] = sub_first; hi[k] = sub_end;         // invariant: prefix(lo) <= pos < prefix(hi)
        }
        bool more = true;
        while (more) {
            more = false;
            u32 mid[8];
            u64 pv[8];
#pragma unroll
            for (u32 k = 0; k < 8; ++k) { mid[k] = (lo[k] + hi[k]) >> 1; pv[k] = pre[mid[k]]; }
#pragma unroll
            for (u32 k = 0; k < 8; ++k) {
                if (hi[k] - lo[k] > 1u) {
                    const u32 at = which == 0 ? (u32)(pv[k] >> 32) : (u32)pv[k];
                    if (at <= pos[k]) lo[k] = mid[k]; else hi[k] = mid[k];
                    more = more || hi[k] - lo[k] > 1u;
                }
            }
        }
#pragma unroll
        for (u32 k = 0; k < 8; ++k) {
            const u32 i = i0 + k * EXCP_THREADS;
            if (i < ns) {
                const u64 pl = pre[lo[k]];
                const u32 at = which == 0 ? (u32)(pl >> 32) : (u32)pl;
                const float v = slots[(u64)(lo[k] - sub_first) * 2048u + (pos[k] - at)];
                smp[i] = v;
                const u32 bits = f2u(v), a = bits & 0x7fffffffu, sg = bits >> 31;
                if (sg) { mn[0] = min(mn[0], a); mx[0] = max(mx[0], a); } else { mn[1] = min(mn[1], a); mx[1] = max(mx[1], a); }
            }
        }
    }
#pragma unroll
    for (int sg = 0; sg < 2; ++sg) {
        u32 lo = mn[sg], hi = mx[sg];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            lo = min(lo, (u32)__shfl_xor(lo, m, WAVE));
            hi = max(hi, (u32)__shfl_xor(hi, m, WAVE));
        }
        if ((tid & 63u) == 0) { atomicMin(&s_ext[2 * sg], lo); atomicMax(&s_ext[2 * sg + 1], hi); }
    }
    __syncthreads();
    if (tid < 2) {
        const u32 lo = s_ext[2 * tid], hi = s_ext[2 * tid + 1];
        u32 amin = 0, sh = 20;                     // no sample of this sign: exponent and 3 mantissa bits
        if (lo <= hi) {
            const u32 width = hi - lo;             // (width >> sh) must stay below 2048
            const u32 bits = width ? 32u - (u32)__clz((int)width) : 0u;
            amin = lo;
            sh = bits > 11u ? bits - 11u : 0u;
        }
        s_map[2 * tid] = amin; s_map[2 * tid + 1] = sh;
    }
    __syncthreads();
    for (u32 i = tid; i < ns; i += EXCP_THREADS) atomicAdd(&cnt[cell_of(smp[i], s_map)], 1u);
    __syncthreads();
    // Exclusive scan over the cells (16 consecutive cells per thread), then bucket = share of the sample
    // below.  A cell that alone holds more than 1/64 of the sample is a tied value (a continuous
    // distribution never fills one of 4096 cells like that): it gets a bucket of its own, so that a bucket
    // is either one repeated value -- which neither the initial order statistics nor the Lloyd
    // iterations ever have to read again -- or an even share of the rest.  With H such cells the others
    // are spread over S = 255 - 2 H buckets; a heavy cell sits one above the light cells before it and
    // one below those after it.
    constexpr u32 PER = EXCP_KM_CELLS / EXCP_THREADS;     // 16
    const u32 heavy_min = max(ns / 64u, 32u);
    u32 local[PER], sum = 0;                               // sum: heavy cells << 16 | samples in light cells
#pragma unroll
    for (u32 q = 0; q < PER; ++q) {
        local[q] = cnt[tid * PER + q];
        sum += local[q] >= heavy_min ? (1u << 16) : local[q];
    }
    s_part[tid] = sum;
    __syncthreads();
    for (u32 off = 1; off < EXCP_THREADS; off <<= 1) {
        const u32 v = (tid >= off) ? s_part[tid - off] : 0u;
        __syncthreads();
        s_part[tid] += v;
        __syncthreads();
    }
    const u32 total = s_part[EXCP_THREADS - 1];
    const u32 H = total >> 16, ns_light = total & 0xffffu;
    const u32 S = NBKT - 1u - 2u * H;                      // H <= 64, so S >= 127
    u32 run = s_part[tid] - sum;
    u32 *out = w.km_split + (u64)sidx * EXCP_KM_MAP_WORDS;
    if (tid < 4) out[tid] = s_map[tid];
#pragma unroll
    for (u32 q4 = 0; q4 < PER / 4; ++q4) {
        u32 word = 0;
#pragma unroll
        for (u32 q = 0; q < 4; ++q) {
            const u32 c = local[q4 * 4 + q];
            const bool heavy = c >= heavy_min;
            const u32 light_before = run & 0xffffu, heavy_before = run >> 16;
            const u32 share = ns_light ? min((u32)(((u64)light_before * S) / ns_light), S - 1u) : 0u;
            const u32 bkt = share + 2u * heavy_before + (heavy ? 1u : 0u);
            word |= bkt << (8u * q);
            run += heavy ? (1u << 16) : c;
        }
        out[4 + tid * (PER / 4) + q4] = word;
    }
}

// Loads the 32 values a thread owns in a chunk: eight groups of four consecutive values (group it
// starts at element (it * 256 + tid) * 4).  Values past the chunk's end are returned as NaN.
__device__ __forceinline__ void load_chunk(const EXCP_GLOBAL float *gx, u32 clen, float (&v)[PER_THREAD]) {
    const u32 tid = threadIdx.x;
    if (clen == EXCP_CHUNK) {
#pragma unroll
        for (u32 it = 0; it < PER_THREAD / 4; ++it) {
            const f4u q = *(const EXCP_GLOBAL f4u *)(gx + (it * EXCP_THREADS + tid) * 4u);
            v[4 * it] = q.x; v[4 * it + 1] = q.y; v[4 * it + 2] = q.z; v[4 * it + 3] = q.w;
        }
    } else {
#pragma unroll
        for (u32 it = 0; it < PER_THREAD; ++it) {
            const u32 e = ((it >> 2) * EXCP_THREADS + tid) * 4u + (it & 3u);
            v[it] = e < clen ? gx[e] : __uint_as_float(0x7fc00000u);
        }
    }
}
__device__ __forceinline__ u32 chunk_elem(u32 it) { return ((it >> 2) * EXCP_THREADS + threadIdx.x) * 4u + (it & 3u); }

// ---------------------------------------------------------------- P1: bucket counts
// Taken by the pass that makes the dense survivor arrays (k_mask_gather), per 16 chunks of a stream, into
// the row of the first of them; the table is cleared here before that pass.
__global__ __launch_bounds__(EXCP_THREADS) void k_km_clear_counts(Workspace w, GroupParams g) {
    const u64 words = (u64)*w.chunk_total * NBKT;
    for (u64 i = (u64)blockIdx.x * EXCP_THREADS + threadIdx.x; i < words; i += (u64)gridDim.x * EXCP_THREADS) w.km_cnt[i] = 0;
}

// ---------------------------------------------------------------- P2: offsets of every (chunk, bucket)
// A stream's chunks are cut into sixteen parts so that sixteen workgroups share the walk over a long
// stream's count table: (a) per-bucket totals of every part, (b) per stream: bucket totals, their
// scan, and the first position of every (part, bucket), (c) per part: counts -> positions.
constexpr u32 SCAN_PARTS = 16;

__device__ __forceinline__ void scan_part_range(const Workspace &w, u32 sidx, u32 part, u32 &a0, u32 &a1) {
    const u32 c0 = w.seg[sidx].chunk_begin, c1 = w.seg_chunk_begin[sidx + 1];
    const u32 per = (c1 - c0 + SCAN_PARTS - 1u) / SCAN_PARTS;
    a0 = min(c0 + part * per, c1);
    a1 = min(a0 + per, c1);
}

// 1024 threads: thread (q, b) owns bucket b over one quarter of the part's chunks.
__global__ __launch_bounds__(1024) void k_km_scan_parts(Workspace w, GroupParams g) {
    __shared__ u32 tot[4][NBKT];
    const u32 sidx = blockIdx.x / SCAN_PARTS, part = blockIdx.x % SCAN_PARTS;
    const u32 tid = threadIdx.x, q = tid >> 8, b = tid & 255u;
    if (w.seg[sidx].len == 0) return;
    u32 p0, p1;
    scan_part_range(w, sidx, part, p0, p1);
    const u32 nq = (p1 - p0 + 3u) / 4u;
    const u32 a0 = min(p0 + q * nq, p1), a1 = min(a0 + nq, p1);
    const u32 *cnt = w.km_cnt;
    u32 s = 0;
#pragma unroll 16
    for (u32 c = a0; c < a1; ++c) s += cnt[(u64)c * NBKT + b];
    tot[q][b] = s;
    __syncthreads();
    if (q == 0) w.km_part[((u64)sidx * SCAN_PARTS + part) * NBKT + b] = tot[0][b] + tot[1][b] + tot[2][b] + tot[3][b];
}

// One workgroup of 256 threads per stream; thread b owns bucket b.
__global__ __launch_bounds__(NBKT) void k_km_scan(Workspace w, GroupParams g) {
    __shared__ u32 begin[NBKT + 1];
    const u32 sidx = blockIdx.x, b = threadIdx.x;
    if (w.seg[sidx].len == 0) return;
    u32 *part = w.km_part + (u64)sidx * SCAN_PARTS * NBKT;
    u32 pt[SCAN_PARTS], total = 0;
#pragma unroll
    for (u32 p = 0; p < SCAN_PARTS; ++p) { pt[p] = part[p * NBKT + b]; total += pt[p]; }
    begin[b + 1] = total;
    if (b == 0) begin[0] = 0;
    __syncthreads();
    // inclusive scan of begin[1..256]
    for (u32 off = 1; off < NBKT; off <<= 1) {
        const u32 v = b >= off ? begin[b + 1 - off] : 0u;
        __syncthreads();
        begin[b + 1] += v;
        __syncthreads();
    }
    w.km_begin[(u64)sidx * (NBKT + 1) + b + 1] = begin[b + 1];
    if (b == 0) w.km_begin[(u64)sidx * (NBKT + 1)] = 0;
    u32 run = begin[b];
#pragma unroll
    for (u32 p = 0; p < SCAN_PARTS; ++p) { part[p * NBKT + b] = run; run += pt[p]; }
}

// 1024 threads: thread (q, b) turns the counts of bucket b into positions over one quarter of the
// part's chunks (its start: the part's first position plus the quarters before it).
__global__ __launch_bounds__(1024) void k_km_scan_apply(Workspace w, GroupParams g) {
    __shared__ u32 tot[4][NBKT];
    const u32 sidx = blockIdx.x / SCAN_PARTS, part = blockIdx.x % SCAN_PARTS;
    const u32 tid = threadIdx.x, q = tid >> 8, b = tid & 255u;
    if (w.seg[sidx].len == 0) return;
    u32 p0, p1;
    scan_part_range(w, sidx, part, p0, p1);
    const u32 nq = (p1 - p0 + 3u) / 4u;
    const u32 a0 = min(p0 + q * nq, p1), a1 = min(a0 + nq, p1);
    u32 *cnt = w.km_cnt;
    u32 s = 0;
#pragma unroll 16
    for (u32 c = a0; c < a1; ++c) s += cnt[(u64)c * NBKT + b];
    tot[q][b] = s;
    __syncthreads();
    u32 run = w.km_part[((u64)sidx * SCAN_PARTS + part) * NBKT + b];
    for (u32 qq = 0; qq < q; ++qq) run += tot[qq][b];
#pragma unroll 16
    for (u32 c = a0; c < a1; ++c) {
        const u32 v = cnt[(u64)c * NBKT + b];
        cnt[(u64)c * NBKT + b] = run;
        run += v;
    }
}

// ---------------------------------------------------------------- P3: scatter into buckets
// A workgroup takes a contiguous range of chunks; inside one stream the runs that consecutive chunks
// contribute to a bucket are neighbours in memory, so the workgroup keeps, per bucket, a ring of up to
// 128 values in LDS and writes a bucket's values as whole, aligned 128-byte lines (partial lines reach
// memory at a fraction of the rate of whole ones: a run of about 32 values that starts anywhere costs
// twice a run that starts on a line).  Partial lines are written only where a workgroup's range or a
// stream begins or ends.  Values arrive 8192 at a time (eight per thread): a value takes the next place
// of its bucket's ring (one LDS atomic on a counter that also carries the ring's read position); then
// thread b looks at bucket b and lists the lines that are complete; then groups of eight lanes write
// the listed lines, sixteen bytes per lane.  A value's ring index is its place inside its memory line,
// so a whole line is one aligned quarter of the ring.  When more values arrive for a bucket in one step
// than its ring holds (tied data: one bucket takes most of a stream), those beyond the ring go straight
// to their places in memory -- consecutive arrivals, consecutive addresses -- and the ring is emptied.
// The order of values inside a bucket is that of arrival, which no reader of a bucket depends on
// (its sum, count, extremes and order statistics are those of a multiset).
constexpr u32 SC_THREADS = 1024, SC_STEP = 8192, SC_PER = SC_STEP / SC_THREADS, SC_RING = 128, SC_LIST = 1536;

__global__ __launch_bounds__(SC_THREADS, 1) void k_km_scatter(Workspace w, GroupParams g) {
    __shared__ __attribute__((aligned(16))) float ring[NBKT][SC_RING];
    __shared__ u32 cells[EXCP_KM_CELLS / 4u];
    __shared__ u32 ctr[NBKT];                            // (ring index of the oldest value) << 16 | values waiting
    __shared__ u32 gpos[NBKT];                           // place of the oldest value in the bucket-ordered array
    __shared__ __attribute__((aligned(8))) u32 list[2 * SC_LIST];   // lines to write: (bucket | ring index << 8 | count << 16), place
    __shared__ u32 nlist;
    const u32 tid = threadIdx.x, grp = tid >> 3, gl = tid & 7u;    // groups of eight lanes write a line each
    const u32 total = *w.chunk_total;
    const u32 G = gridDim.x, bid = blockIdx.x;
    const u32 nseg = 3u * g.ntensors;
    // Equal shares of the chunk list, their ends moved back to where the bucket counts were taken: the first
    // of every 16 chunks of a stream (the counts of a unit sit in that chunk's row, the rows between are zero).
    auto snapped = [&](u32 c) -> u32 {
        if (c >= total) return total;
        const u32 c0 = w.seg_chunk_begin[find_owner(w.seg_chunk_begin, nseg, c)];
        return c0 + ((c - c0) & ~(EXCP_SUPER_CHUNKS - 1u));
    };
    const u32 lo = snapped((u32)(((u64)bid * total) / G)), hi = snapped((u32)(((u64)(bid + 1) * total) / G));
    if (lo >= hi) return;
    if (tid == 0) nlist = 0;

    for (u32 c = lo; c < hi;) {
        // the chunks [c, c_end) of this workgroup that belong to one stream
        __syncthreads();
        const u32 sidx = find_owner(w.seg_chunk_begin, nseg, c);
        const u32 c_end = min(hi, w.seg_chunk_begin[sidx + 1]);
        const u64 len = w.seg[sidx].len;
        const u32 chunk0 = w.seg[sidx].chunk_begin;
        const EXCP_GLOBAL float *data = gptr(seg_data(w, sidx));
        EXCP_GLOBAL float *part = gptr(seg_part(w, sidx));
        const u32 misalign = (u32)(((uintptr_t)seg_part(w, sidx) >> 2) & 31u);   // (place + misalign) % 32 == 0: a line starts
        // the value -> bucket table stays in global memory (4 KB, read through the vector cache): the LDS unit
        // is what this kernel is short of
        const u32 *mp = w.km_split + (u64)sidx * EXCP_KM_MAP_WORDS;
        const u32 neg_min = mp[0], neg_sh = mp[1], pos_min = mp[2], pos_sh = mp[3];
        for (u32 i = tid; i < EXCP_KM_CELLS / 4u; i += SC_THREADS) cells[i] = mp[4u + i];
        const unsigned char *cellmap = (const unsigned char *)cells;
        auto bucket = [&](float x) -> u32 {
            const u32 bits = f2u(x), a = bits & 0x7fffffffu;
            const bool neg = bits >> 31;
            const u32 amin = neg ? neg_min : pos_min, sh = neg ? neg_sh : pos_sh;
            const u32 cc = min((max(a, amin) - amin) >> sh, HALF_CELLS - 1u);
            return cellmap[neg ? (cc ^ (HALF_CELLS - 1u)) : (cc | HALF_CELLS)];
        };
        if (tid < NBKT) {
            // a ring index is the value's place inside its line, so that whole lines sit in one quarter of the ring
            const u32 gp = w.km_cnt[(u64)c * NBKT + tid];
            gpos[tid] = gp;
            ctr[tid] = ((gp + misalign) & 31u) << 16;
        }
        const u64 e_begin = (u64)(c - chunk0) * EXCP_CHUNK;
        const u64 e_stop = min(len, (u64)(c_end - chunk0) * EXCP_CHUNK);
        __syncthreads();

        // thread b: which lines of bucket b can be written now (at the end of the range: everything)
        auto plan = [&](bool final) {
            if (tid >= NBKT) return;                    // (whole waves)
            const u32 b = tid;
            const u32 cv = ctr[b];
            const u32 arrived = cv & 0xffffu;           // since the last look: more than the ring holds if the bucket is crowded
            const bool over = arrived > SC_RING;        // the values beyond the ring went straight to their places
            const bool all = final || over;
            const u32 f0 = min(arrived, SC_RING), h0 = cv >> 16, gp0 = gpos[b];
            // what leaves: the values up to the next line start, then whole lines, and (all) the rest
            const u32 mis = (gp0 + misalign) & 31u;
            u32 f = f0, head_cnt = 0;
            if (f && mis && (f >= 32u - mis || all)) { head_cnt = min(32u - mis, f); f -= head_cnt; }
            const bool aligned = ((gp0 + head_cnt + misalign) & 31u) == 0u;
            const u32 nfull = aligned ? f >> 5 : 0u;
            f -= nfull << 5;
            const u32 tail_cnt = (aligned && all) ? f : 0u;
            f -= tail_cnt;
            const u32 ne = (head_cnt ? 1u : 0u) + nfull + (tail_cnt ? 1u : 0u);
            const u32 gone = f0 - f;
            if (over) {                                 // the ring is empty and starts again behind everything that arrived
                gpos[b] = gp0 + arrived;
                ctr[b] = ((gp0 + arrived + misalign) & 31u) << 16;
            } else {
                ctr[b] = (((h0 + gone) & (SC_RING - 1u)) << 16) | f; gpos[b] = gp0 + gone;
            }
            // places in the list: one atomic per wave, the lanes' shares by counting the set bits below them
            const u64 b0 = ballot64(ne & 1u), b1 = ballot64(ne & 2u), b2 = ballot64(ne & 4u);
            const u32 wave_total = (u32)__popcll(b0) + 2u * (u32)__popcll(b1) + 4u * (u32)__popcll(b2);
            if (wave_total) {
                u32 base = 0;
                if ((tid & 63u) == 0u) base = atomicAdd(&nlist, wave_total);
                base = (u32)__builtin_amdgcn_readfirstlane((int)base);
                u32 at = base + lanes_below(b0) + 2u * lanes_below(b1) + 4u * lanes_below(b2);
                u32 h = h0, gp = gp0;
                auto emit = [&](u32 cnt) {
                    list[2u * at] = b | (h << 8) | (cnt << 16); list[2u * at + 1u] = gp; ++at;
                    h = (h + cnt) & (SC_RING - 1u); gp += cnt;
                };
                if (head_cnt) emit(head_cnt);
                for (u32 k = 0; k < nfull; ++k) emit(32u);
                if (tail_cnt) emit(tail_cnt);
            }
        };
        // groups of eight lanes write the listed lines, four values per lane
        auto write_lines = [&]() {
            const u32 n = nlist;
            constexpr u32 GROUPS = SC_THREADS / 8u;
            for (u32 i = grp; i < n; i += GROUPS) {
                const u64 ev = *(const u64 *)&list[2u * i];
                const u32 e0 = (u32)ev, b = e0 & 255u, off = (e0 >> 8) & 255u, cnt = e0 >> 16, gp = (u32)(ev >> 32);
                if (cnt == 32u) {                       // a whole line: it sits in one half of the ring, and on a line in memory
                    typedef float f4a __attribute__((ext_vector_type(4)));      // 16-byte aligned on both sides
                    const f4a x = *(const f4a *)&ring[b][off + 4u * gl];
                    *(EXCP_GLOBAL f4a *)(part + (u64)gp + 4u * gl) = x;
                } else {
#pragma unroll
                    for (u32 k = 0; k < 4; ++k) {
                        const u32 idx = 4u * gl + k;
                        if (idx < cnt) part[(u64)gp + idx] = ring[b][(off + idx) & (SC_RING - 1u)];
                    }
                }
            }
        };

        float nx[SC_PER];
        auto load_step = [&](u64 e, float (&v)[SC_PER]) {
            const u32 nval = (e_stop - e) < (u64)SC_STEP ? (u32)(e_stop - e) : SC_STEP;
            if (nval == SC_STEP) {
#pragma unroll
                for (u32 q = 0; q < SC_PER / 4; ++q) {
                    const f4u x = *(const EXCP_GLOBAL f4u *)(data + e + (q * SC_THREADS + tid) * 4u);
                    v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
                }
            } else {
#pragma unroll
                for (u32 j = 0; j < SC_PER; ++j) {
                    const u32 el = ((j >> 2) * SC_THREADS + tid) * 4u + (j & 3u);
                    v[j] = el < nval ? data[e + el] : 0.f;
                }
            }
        };
        if (e_begin < e_stop) load_step(e_begin, nx);
        for (u64 e = e_begin; e < e_stop; e += SC_STEP) {
            const u32 nval = (e_stop - e) < (u64)SC_STEP ? (u32)(e_stop - e) : SC_STEP;
            float v[SC_PER];
#pragma unroll
            for (u32 j = 0; j < SC_PER; ++j) v[j] = nx[j];
            if (e + SC_STEP < e_stop) load_step(e + SC_STEP, nx);      // the next step's values are on their way
            u32 bb[SC_PER], cv[SC_PER];
#pragma unroll
            for (u32 j = 0; j < SC_PER; ++j) bb[j] = bucket(v[j]);
            if (tid == 0) nlist = 0;
            // a value takes the next place of its bucket: in the ring, or, when more than the ring holds have
            // arrived since the bucket was last looked at (tied data: one bucket takes most of a stream),
            // straight in the bucket-ordered array
            if (nval == SC_STEP) {
#pragma unroll
                for (u32 j = 0; j < SC_PER; ++j) cv[j] = atomicAdd(&ctr[bb[j]], 1u);
#pragma unroll
                for (u32 j = 0; j < SC_PER; ++j) {
                    const u32 pos = cv[j] & 0xffffu;
                    if (pos < SC_RING) ring[bb[j]][((cv[j] >> 16) + pos) & (SC_RING - 1u)] = v[j];
                    else part[(u64)gpos[bb[j]] + pos] = v[j];
                }
            } else {
#pragma unroll
                for (u32 j = 0; j < SC_PER; ++j) {
                    if (((j >> 2) * SC_THREADS + tid) * 4u + (j & 3u) < nval) {
                        const u32 c1 = atomicAdd(&ctr[bb[j]], 1u), pos = c1 & 0xffffu;
                        if (pos < SC_RING) ring[bb[j]][((c1 >> 16) + pos) & (SC_RING - 1u)] = v[j];
                        else part[(u64)gpos[bb[j]] + pos] = v[j];
                    }
                }
            }
            __syncthreads();
            plan(false);
            __syncthreads();
            write_lines();
            __syncthreads();
        }
        // the end of the stream or of this workgroup's range: what is left goes out as it is
        if (tid == 0) nlist = 0;
        __syncthreads();
        plan(true);
        __syncthreads();
        write_lines();
        c = c_end;
    }
}

// ---------------------------------------------------------------- P4: exact totals per bucket
// One workgroup per four buckets of a stream (per bucket in the sixteen-wave form); its waves share every bucket,
// so that one very large bucket (tied values) does not leave a single wave working alone.  Values of a bucket
// are neighbours in value, hence in exponent: a window of 24 bit positions placed from the first
// values met holds practically all of them; inside it a lane adds sixteen values at a time exactly in
// fp64 and keeps the running total in two integer counters, with no cross-lane traffic; the rest
// (rare) is filed one by one.
// (sixteen for 16-bit weights, whose residuals are heavily tied, and for groups with a tensor so large
// that its buckets alone are millions of values; four otherwise, which is faster when the buckets are
// small and even)
template <u32 BS_WAVES, u32 BPW>
__global__ __launch_bounds__(BS_WAVES * 64) void k_km_bucket_stats(Workspace w, GroupParams g) {
    __shared__ u64 bins[BPW][EXCP_ABSM_BINS];
    __shared__ u32 s_min[BPW], s_max[BPW];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 nseg = 3u * g.ntensors;
    // a workgroup walks over sets of BPW buckets (many sets are tiny: one workgroup each would be
    // bound by the rate at which workgroups can be started)
    for (u64 first = (u64)blockIdx.x * BPW; first < (u64)nseg * NBKT; first += (u64)gridDim.x * BPW) {
    const u32 sidx = (u32)(first / NBKT), b0 = (u32)(first % NBKT);
    if (w.seg[sidx].len == 0) continue;                    // the same for the whole workgroup
    __syncthreads();                                       // the previous set has left the LDS tables
    if (tid < BPW * EXCP_ABSM_BINS) (&bins[0][0])[tid] = 0;
    if (tid < BPW) { s_min[tid] = 0xffffffffu; s_max[tid] = 0; }
    __syncthreads();
    const u32 *begin = w.km_begin + (u64)sidx * (NBKT + 1);
    const EXCP_GLOBAL float *part = gptr(seg_part(w, sidx));
    // Small buckets (the four together at most SOLO_MAX values: small tensors, small models): a wave
    // takes a whole bucket, the four side by side, instead of four rounds of memory round trips.
    constexpr u32 SOLO_MAX = 4096;
    const bool solo = BS_WAVES == BPW && begin[b0 + BPW] - begin[b0] <= SOLO_MAX;
    for (u32 jj = 0; jj < (solo ? 1u : BPW); ++jj) {
        const u32 j = solo ? wave : jj;
        const u32 q0 = begin[b0 + j], q1 = begin[b0 + j + 1];
        // this wave's share, cut at multiples of 256 values from the bucket's start
        const u32 blocks = (q1 - q0 + 255u) >> 8, per = (blocks + BS_WAVES - 1u) / BS_WAVES;
        const u32 p0 = solo ? q0 : min(q0 + wave * per * 256u, q1), p1 = solo ? q1 : min(p0 + per * 256u, q1);
        if (p0 >= p1) continue;
        u64 *mybins = bins[j];
        // window base from the first (up to) 64 values: top 4 binary orders above their largest
        u32 pm = 0;
        {
            const u32 i = p0 + lane;
            const u32 mb = (i < p1) ? (f2u(part[i]) & 0x7fffffffu) : 0u;
            const u32 e = mb >> 23;
            pm = wave_max_u32((e ? e : 1u) - 1u);
        }
        const u32 B = pm + 4u > 23u ? pm + 4u - 23u : 0u;
        u32 thr_lo, span;
        window_range(B, thr_lo, span);
        WindowSum S;
        u32 kmin = 0xffffffffu, kmax = 0;
        // Tied data (the sixteen-wave form): a large bucket is mostly one value.  The wave takes its
        // first value as that one and only counts its repetitions; count times value joins the sums
        // at the end.
        u32 dom = 0xffffffffu, ndom = 0;                   // bit pattern of the repeated value; this lane's count
        if (BS_WAVES == 16u) {
            const u32 head = f2u(part[p0]);
            if ((head & 0x7fffffffu) - thr_lo < span && (head & 0x7fffffffu)) dom = head;     // inside the window, not zero
        }
        auto take = [&](float xv) {
            const u32 u = f2u(xv), mb = u & 0x7fffffffu;
            if (BS_WAVES == 16u && u == dom) { ++ndom; return; }
            const u32 k = key_of(xv);
            kmin = min(kmin, k); kmax = max(kmax, k);
            if (mb - thr_lo < span) {
                S.part += (double)xv;
            } else if (mb) {
                const u32 e = mb >> 23;
                const u32 mant = (mb & 0x7fffffu) | (e ? 0x800000u : 0u);
                const u32 pos = (e ? e : 1u) - 1u;
                const u64 d = (u64)mant << (pos & 7u);
                atomicAdd(&mybins[pos >> 3], (u >> 31) ? (u64)0 - d : d);
            }
        };
        // four 16-byte loads in flight per lane: the share of a wave in a large bucket is a chain of
        // round trips otherwise.  Sixteen values per round: one fold of the fp64 partial sum.
        u32 p = p0;
        for (; p + 1024u <= p1; p += 1024u) {
            f4u q[4];
#pragma unroll
            for (u32 r = 0; r < 4; ++r) q[r] = *(const EXCP_GLOBAL f4u *)(part + p + r * 256u + lane * 4u);
#pragma unroll
            for (u32 r = 0; r < 4; ++r) { take(q[r].x); take(q[r].y); take(q[r].z); take(q[r].w); }
            S.fold(B);
        }
        for (; p < p1; p += 256u) {                       // (at most four rounds of four values)
            const u32 i = p + lane * 4u;
            if (p + 256u <= p1) {
                const f4u q = *(const EXCP_GLOBAL f4u *)(part + i);
                take(q.x); take(q.y); take(q.z); take(q.w);
            } else {
#pragma unroll
                for (u32 e = 0; e < 4; ++e) if (i + e < p1) take(part[i + e]);
            }
        }
        S.fold(B);
        if (BS_WAVES == 16u && ndom) {
            const u32 mb = dom & 0x7fffffffu, e = mb >> 23;
            const u32 mant = (mb & 0x7fffffu) | (e ? 0x800000u : 0u);
            const u64 term = (u64)mant << (((e ? e : 1u) - 1u) - B);                      // below 2^47 units
            const long long tl = (long long)((term & 0xffffffffull) * ndom), th = (long long)((term >> 32) * ndom);   // a lane sees < 2^20 values
            if (dom >> 31) { S.lo -= tl; S.hi -= th; } else { S.lo += tl; S.hi += th; }
            const u32 k = key_of(u2f(dom));
            kmin = min(kmin, k); kmax = max(kmax, k);
        }
        const long long tL = (long long)wave_sum_u64((u64)S.lo), tH = (long long)wave_sum_u64((u64)S.hi);
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            kmin = min(kmin, (u32)__shfl_xor(kmin, m, WAVE));
            kmax = max(kmax, (u32)__shfl_xor(kmax, m, WAVE));
        }
        if (lane == 0) {
            atomicMin(&s_min[j], kmin); atomicMax(&s_max[j], kmax);
            file_i64(mybins, tL, B); file_i64(mybins, tH, B + 32u);
        }
    }
    __syncthreads();
    if (tid < BPW * EXCP_ABSM_BINS)
        w.km_bsum[((u64)sidx * NBKT + b0) * EXCP_ABSM_BINS + tid] = (&bins[0][0])[tid];
    if (tid < BPW) { w.km_min[(u64)sidx * NBKT + b0 + tid] = s_min[tid]; w.km_max[(u64)sidx * NBKT + b0 + tid] = s_max[tid]; }
    if (BS_WAVES != 4u) break;                             // the sixteen-wave forms are launched one workgroup per set
    }
}

// ---------------------------------------------------------------- P6: initial centres
// One workgroup per (stream, rank): radix select inside the bucket that holds the rank; the bits
// that the bucket's minimum and maximum key share are known and skipped.
// (1024 threads for 16-bit weights -- a bucket of tied values can be most of a stream -- and for very
// large tensors; 256 otherwise)
template <u32 INIT_THREADS>
__global__ __launch_bounds__(INIT_THREADS) void k_km_init(Workspace w, GroupParams g) {
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
    const EXCP_GLOBAL float *gpart = gptr(seg_part(w, sidx));
    u32 diff = kmin ^ kmax;
    if (diff == 0) { if (tid == 0) S.C[k] = val_of(kmin); return; }
    // A bucket far above the average size holds tied values (a continuous distribution fills the
    // buckets evenly).  Such a bucket is mostly ONE value, its smallest or its largest key, with a few
    // strays beside it: one cheap pass counts the two extremes, and if the rank falls among them the
    // answer is known without any digit-by-digit selection.
    const bool crowded = (u64)(p1 - p0) > 3ull * (len / NBKT + 1ull);
    if (crowded) {
        __shared__ u32 s_ext[2];
        if (tid == 0) { s_ext[0] = 0u; s_ext[1] = 0u; }
        __syncthreads();
        u32 c_lo = 0, c_hi = 0;
        for (u32 q0 = p0; q0 < p1; q0 += 16u * INIT_THREADS) {
            if (q0 + 16u * INIT_THREADS <= p1) {
                f4u q[4];
#pragma unroll
                for (u32 j = 0; j < 4; ++j) q[j] = *(const EXCP_GLOBAL f4u *)(gpart + q0 + (j * INIT_THREADS + tid) * 4u);
#pragma unroll
                for (u32 j = 0; j < 4; ++j) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const u32 key = key_of(q[j][e]);
                        c_lo += key == kmin; c_hi += key == kmax;
                    }
                }
            } else {
                for (u32 p = q0 + tid; p < p1; p += INIT_THREADS) {
                    const u32 key = key_of(gpart[p]);
                    c_lo += key == kmin; c_hi += key == kmax;
                }
            }
        }
        c_lo = wave_sum_u32(c_lo); c_hi = wave_sum_u32(c_hi);
        if ((tid & 63u) == 0u) { atomicAdd(&s_ext[0], c_lo); atomicAdd(&s_ext[1], c_hi); }
        __syncthreads();
        if (rank < s_ext[0]) { if (tid == 0) S.C[k] = val_of(kmin); return; }
        if (rank >= (p1 - p0) - s_ext[1]) { if (tid == 0) S.C[k] = val_of(kmax); return; }
    }
    int hb = 31 - __clz((int)diff);          // highest bit in which keys of this bucket differ
    u32 prefix = kmin >> (hb + 1 > 31 ? 31 : hb + 1);
    if (hb == 31) prefix = 0;
    int top = hb;                            // bits [0, top] still unknown
    while (top >= 0) {
        const int width = top + 1 < 8 ? top + 1 : 8;
        const int shift = top + 1 - width;
        if (tid < 256u) hist[tid] = 0;
        __syncthreads();
        // (in a crowded bucket the lanes mostly hit the same bin: the increments are grouped per wave)
        auto tally = [&](float xv, bool in) {
            const u32 key = key_of(xv);
            const bool match = in && ((top == 31) ? true : ((key >> (top + 1)) == prefix));
            const u32 bin = (key >> shift) & ((1u << width) - 1u);
            if (crowded) hist_add_tied(hist, bin, match);
            else if (match) atomicAdd(&hist[bin], 1u);
        };
        // sixteen values per thread and round, every load of a round issued before its use
        for (u32 q0 = p0; q0 < p1; q0 += 16u * INIT_THREADS) {
            if (q0 + 16u * INIT_THREADS <= p1) {
                f4u q[4];
#pragma unroll
                for (u32 j = 0; j < 4; ++j) q[j] = *(const EXCP_GLOBAL f4u *)(gpart + q0 + (j * INIT_THREADS + tid) * 4u);
#pragma unroll
                for (u32 j = 0; j < 4; ++j) { tally(q[j].x, true); tally(q[j].y, true); tally(q[j].z, true); tally(q[j].w, true); }
            } else {
                for (u32 pp = q0; pp < p1; pp += INIT_THREADS) {       // the same trip count in every lane
                    const u32 p = pp + tid;
                    tally(p < p1 ? gpart[p] : 0.f, p < p1);
                }
            }
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

// New centres of one stream from the iteration's totals: centre = fp32(exact sum / count), a
// cluster without members keeps its centre; then the centres are put back in ascending order; the
// totals are cleared for the next iteration.
// Called by the whole workgroup (it holds barriers); the totals of sixteen centres at a time are
// fetched into LDS side by side, so that no thread walks a chain of dependent global reads.
// lds_C (optional) receives the centres as well.
__device__ __forceinline__ void move_centres(const Workspace &w, const GroupParams &g, u32 sidx, float *lds_C) {
    constexpr u32 STRIDE = EXCP_ABSM_BINS + 1, BATCH = 16;
    __shared__ u64 s_acc[BATCH * STRIDE];
    __shared__ float s_new[EXCP_MAX_K + 1];
    SegState &S = w.seg[sidx];
    const u32 K = (u32)g.K, tid = threadIdx.x;
    u64 *acc = w.km_acc + (u64)sidx * EXCP_MAX_K * STRIDE;
    for (u32 k0 = 0; k0 < K; k0 += BATCH) {
        const u32 nk = min(BATCH, K - k0);
        __syncthreads();
        for (u32 i = tid; i < nk * STRIDE; i += EXCP_THREADS) {
            s_acc[i] = acc[(u64)k0 * STRIDE + i];
            acc[(u64)k0 * STRIDE + i] = 0;
        }
        __syncthreads();
        if (tid < nk) {
            const u64 *a = s_acc + tid * STRIDE;
            const u64 cnt = a[EXCP_ABSM_BINS];
            float c = S.C[k0 + tid];
            if (cnt) {
                const double sum = signed_bins_to_double(a);
                c = (float)(sum / (double)cnt);
            }
            s_new[k0 + tid] = c;
        }
    }
    __syncthreads();
    // Back into ascending order (stable; nothing moves unless a run of equal centres was torn apart:
    // the lowest of them takes all their members and may pass the ones left behind).
    float c = 0.f; u32 rank = 0;
    if (tid < K) {
        c = s_new[tid];
        for (u32 j = 0; j < K; ++j) {
            const float cj = s_new[j];
            rank += (cj < c || (cj == c && j < tid)) ? 1u : 0u;
        }
    }
    __syncthreads();
    if (tid < K) {
        S.C[rank] = c;
        if (lds_C) lds_C[rank] = c;
    }
}

// ---------------------------------------------------------------- P5a: one Lloyd accumulation
// Classification (one workgroup per stream): every bucket is compared with the current centres.
// A bucket whose smallest and largest value go to the same centre adds its stored totals to that
// centre; a bucket that a cluster border cuts is split into work items of at most 16384 values.
constexpr u32 KM_ITEM = 16384;                   // values per work item
struct KmItem { u32 sidx, p0, p1, range; };      // range = alo | ahi << 8

__global__ __launch_bounds__(EXCP_THREADS) void k_km_classify(Workspace w, GroupParams g, u32 parity, u32 do_update) {
    __shared__ float s_C[EXCP_MAX_K + 1];
    __shared__ u32 s_cut[EXCP_MAX_K + 1];
    __shared__ u32 s_scan[EXCP_THREADS];
    __shared__ u32 s_base;
    const u32 sidx = blockIdx.x, tid = threadIdx.x;
    SegState &S = w.seg[sidx];
    // the work list of the next iteration (the other of two) starts empty; nobody reads it now
    if (sidx == 0 && tid == 0) w.km_item_count[parity ^ 1u] = 0;
    if (S.len == 0) return;
    const int K = g.K;
    u32 kp2 = 1; while (kp2 < (u32)K) kp2 <<= 1;
    if (do_update) move_centres(w, g, sidx, s_C);          // the previous iteration's totals
    else for (u32 k = tid; k < (u32)K; k += EXCP_THREADS) s_C[k] = S.C[k];
    __syncthreads();
    compute_cut_keys(s_C, K, s_cut);
    __syncthreads();
    if (tid >= 1) S.cut[tid] = s_cut[tid];
    const u32 *begin = w.km_begin + (u64)sidx * (NBKT + 1);
    u64 *acc = w.km_acc + (u64)sidx * EXCP_MAX_K * (EXCP_ABSM_BINS + 1);     // [K][bins + count]
    const u32 b = tid;
    const u32 p0 = begin[b], p1 = begin[b + 1], cntb = p1 - p0;
    u32 alo = 0, ahi = 0;
    if (cntb) {
        alo = centre_by_cuts(s_cut, kp2, w.km_min[(u64)sidx * NBKT + b]);
        ahi = centre_by_cuts(s_cut, kp2, w.km_max[(u64)sidx * NBKT + b]);
    }
    const bool cut = cntb && alo != ahi;
    if (cntb && !cut) {
        u64 *dst = acc + (u64)alo * (EXCP_ABSM_BINS + 1);
        const u64 *src = w.km_bsum + ((u64)sidx * NBKT + b) * EXCP_ABSM_BINS;
        u64 tot[EXCP_ABSM_BINS];                   // all reads first: they must not queue behind the atomics
#pragma unroll
        for (int q = 0; q < EXCP_ABSM_BINS; ++q) tot[q] = src[q];
#pragma unroll
        for (int q = 0; q < EXCP_ABSM_BINS; ++q) if (tot[q]) atomicAdd(&dst[q], tot[q]);
        atomicAdd(&dst[EXCP_ABSM_BINS], (u64)cntb);
    }
    const u32 nitems = cut ? (cntb + KM_ITEM - 1) / KM_ITEM : 0u;
    s_scan[tid] = nitems;
    __syncthreads();
    for (u32 off = 1; off < EXCP_THREADS; off <<= 1) {
        u32 v = (tid >= off) ? s_scan[tid - off] : 0u;
        __syncthreads();
        s_scan[tid] += v;
        __syncthreads();
    }
    if (tid == EXCP_THREADS - 1) s_base = s_scan[tid] ? atomicAdd(&w.km_item_count[parity], s_scan[tid]) : 0u;
    __syncthreads();
    u32 at = s_base + s_scan[tid] - nitems;
    KmItem *items = (KmItem *)w.km_items;
    for (u32 q = 0; q < nitems; ++q, ++at) {
        if (at >= w.km_item_cap) { atomicExch(w.err_flag, 1); break; }
        u32 a0 = p0 + q * KM_ITEM, a1 = a0 + KM_ITEM < p1 ? a0 + KM_ITEM : p1;
        items[at] = KmItem{sidx, a0, a1, alo | (ahi << 8)};
    }
}

// Work items: the values of a cut bucket are assigned one by one and added, exactly, to their
// centres.  Sums are gathered in LDS per item and flushed with a few integer atomics.
constexpr u32 ITEM_R = 8;      // centres per item held in LDS; wider ranges go straight to global memory

__global__ __launch_bounds__(EXCP_THREADS, 4) void k_km_iter(Workspace w, GroupParams g, u32 parity) {
    __shared__ float s_C[EXCP_MAX_K + 1];
    __shared__ u32 s_cut[EXCP_MAX_K + 1];
    __shared__ u64 s_bins[ITEM_R][EXCP_ABSM_BINS + 1];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int K = g.K;
    u32 kp2 = 1; while (kp2 < (u32)K) kp2 <<= 1;
    u32 nitems = w.km_item_count[parity];
    if (nitems > w.km_item_cap) nitems = w.km_item_cap;
    const KmItem *items = (const KmItem *)w.km_items;
    u32 cur = 0xffffffffu;
    for (u32 it = blockIdx.x; it < nitems; it += gridDim.x) {
        const KmItem I = items[it];
        const u32 c_lo = I.range & 255u, c_hi = I.range >> 8;
        u64 *acc = w.km_acc + (u64)I.sidx * EXCP_MAX_K * (EXCP_ABSM_BINS + 1);
        if (c_hi - c_lo <= 2u) {
            // ---- one or two borders inside the item (the usual case): per-lane totals of all values and
            // of the values at or above each border; cluster totals are differences.
            // A value inside the window of 24 bit positions [B, B + 24) is a whole multiple of the unit
            // 2^(B-149) below 2^47 units, so a lane adds sixteen of them (one round of loads) exactly in
            // fp64, whatever their signs; the round's sum is then split into two integers (units below
            // 2^32, and signed multiples of 2^32) that go on in integer counters.  Values outside the
            // window (rare: a bucket's values are neighbours) are filed one by one.
            const u32 cut1 = w.seg[I.sidx].cut[c_lo + 1];
            const u32 cut2 = (c_hi - c_lo == 2u) ? w.seg[I.sidx].cut[c_lo + 2] : 0xffffffffu;
            const EXCP_GLOBAL float *part = gptr(seg_part(w, I.sidx));
            const u32 blocks = (I.p1 - I.p0 + 255u) >> 8, per = (blocks + 3u) >> 2;
            const u32 p0 = min(I.p0 + wave * per * 256u, I.p1), p1 = min(p0 + per * 256u, I.p1);
            if (p0 >= p1) continue;                        // nothing for this wave (no barrier on this path)
            u32 pm = 0;
            {
                const u32 i = p0 + lane;
                const u32 mb = (i < p1) ? (f2u(part[i]) & 0x7fffffffu) : 0u;
                const u32 e = mb >> 23;
                pm = wave_max_u32((e ? e : 1u) - 1u);
            }
            const u32 B = pm + 4u > 23u ? pm + 4u - 23u : 0u;       // the window's top: 4 binary orders above the first values
            u32 thr_lo, span;
            window_range(B, thr_lo, span);
            WindowSum S[3];                                // [0] all values, [1] values at or above border 1, [2] at or above border 2
            u32 cnt1 = 0, cnt2 = 0;
            auto take = [&](float xv) {
                const u32 u = f2u(xv), mb = u & 0x7fffffffu;
                const u32 key = key_of(xv);
                const bool up1 = key >= cut1, up2 = key >= cut2;
                cnt1 += up1; cnt2 += up2;
                if (mb - thr_lo < span) {
                    const double xd = (double)xv;
                    S[0].part += xd; S[1].part += up1 ? xd : 0.0; S[2].part += up2 ? xd : 0.0;
                } else if (mb) {
                    const u32 e = mb >> 23;
                    const u32 mant = (mb & 0x7fffffu) | (e ? 0x800000u : 0u);
                    const u32 pos = (e ? e : 1u) - 1u;
                    const u64 dd = (u64)mant << (pos & 7u);
                    const u32 cl = c_lo + (up1 ? 1u : 0u) + (up2 ? 1u : 0u);
                    atomicAdd(&acc[(u64)cl * (EXCP_ABSM_BINS + 1) + (pos >> 3)], (u >> 31) ? (u64)0 - dd : dd);
                }
            };
            auto flush = [&]() { S[0].fold(B); S[1].fold(B); S[2].fold(B); };     // after at most sixteen values
            // four 16-byte loads in flight per lane
            constexpr u32 LOADS = 4;
            u32 p = p0;
            for (; p + LOADS * 256u <= p1; p += LOADS * 256u) {
                f4u q[LOADS];
#pragma unroll
                for (u32 j = 0; j < LOADS; ++j) q[j] = *(const EXCP_GLOBAL f4u *)(part + p + j * 256u + lane * 4u);
#pragma unroll
                for (u32 j = 0; j < LOADS; ++j) { take(q[j].x); take(q[j].y); take(q[j].z); take(q[j].w); }
                flush();
            }
            for (u32 n4 = 0; p < p1; p += 256u) {
                const u32 i = p + lane * 4u;
                if (p + 256u <= p1) {
                    const f4u q = *(const EXCP_GLOBAL f4u *)(part + i);
                    take(q.x); take(q.y); take(q.z); take(q.w);
                } else {
#pragma unroll
                    for (u32 e = 0; e < 4; ++e) if (i + e < p1) take(part[i + e]);
                }
                if (++n4 == 4u) { flush(); n4 = 0; }
            }
            flush();
            long long tL[3], tH[3];
#pragma unroll
            for (int s3 = 0; s3 < 3; ++s3) { tL[s3] = (long long)wave_sum_u64((u64)S[s3].lo); tH[s3] = (long long)wave_sum_u64((u64)S[s3].hi); }
            cnt1 = wave_sum_u32(cnt1); cnt2 = wave_sum_u32(cnt2);
            if (lane == 0) {
                // cluster c_lo + j receives set j minus set j + 1
                const u32 cnt[4] = {p1 - p0, cnt1, cnt2, 0u};
#pragma unroll
                for (u32 j = 0; j < 3; ++j) {
                    if (c_lo + j > c_hi) break;
                    u64 *dst = acc + (u64)(c_lo + j) * (EXCP_ABSM_BINS + 1);
                    file_i64(dst, tL[j], B); file_i64(dst, tH[j], B + 32u);
                    if (j < 2 && c_lo + j < c_hi) { file_i64(dst, -tL[j + 1], B); file_i64(dst, -tH[j + 1], B + 32u); }
                    const u32 nxt = (c_lo + j < c_hi) ? cnt[j + 1] : 0u;
                    if (cnt[j] - nxt) atomicAdd(&dst[EXCP_ABSM_BINS], (u64)(cnt[j] - nxt));
                }
            }
            continue;
        }
        // ---- three or more borders inside one item (degenerate data): per-cluster accumulation
        __syncthreads();
        if (I.sidx != cur) {
            for (u32 k = tid; k < (u32)K; k += EXCP_THREADS) s_C[k] = w.seg[I.sidx].C[k];
            for (u32 k = tid; k <= EXCP_MAX_K; k += EXCP_THREADS) s_cut[k] = w.seg[I.sidx].cut[k];
            cur = I.sidx;
        }
        for (u32 i = tid; i < ITEM_R * (EXCP_ABSM_BINS + 1); i += EXCP_THREADS) (&s_bins[0][0])[i] = 0;
        __syncthreads();
        const bool in_lds = (c_hi - c_lo) < ITEM_R;
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
            for (int j = 0; j < 8; ++j) a[j] = ok[j] ? centre_by_cuts(s_cut, kp2, key_of(x[j])) : 0xffffffffu;
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
// After the last iteration (earlier ones are moved by the next classification kernel).
__global__ __launch_bounds__(EXCP_THREADS) void k_km_update(Workspace w, GroupParams g) {
    const u32 sidx = blockIdx.x, tid = threadIdx.x;
    if (sidx == 0 && tid < 2) w.km_item_count[tid] = 0;    // both work lists start empty next time
    if (w.seg[sidx].len == 0) return;
    move_centres(w, g, sidx, nullptr);
}

// The codes of a thread's 32 values of a whole chunk, ORed into the chunk's bit stream in LDS; returns
// the thread's share of the objective.  The four values of a group go through the bisection over the
// cut keys side by side, so that four table reads are in flight at every step instead of one.
__device__ __forceinline__ double assign_whole_chunk(const float (&v)[PER_THREAD], const u32 *s_cut, const float *s_C, u32 kp2,
                                                     u32 nbits, u32 *s_pack) {
    double obj = 0.0;
    u32 tid = threadIdx.x;
    asm volatile("" : "+v"(tid));                  // bit positions are worked out where they are used, not kept from chunk to chunk
    const unsigned char *cut_b = (const unsigned char *)s_cut, *cen_b = (const unsigned char *)s_C;
#pragma unroll
    for (u32 q = 0; q < PER_THREAD / 4; ++q) {
        u32 key[4], p4[4];                         // p4: four times the number of cut keys <= key found so far (a byte offset)
#pragma unroll
        for (u32 j = 0; j < 4; ++j) { key[j] = key_of(v[4 * q + j]); p4[j] = 0; }
        for (u32 step4 = kp2 << 1; step4 >= 4u; step4 >>= 1) {  // as centre_by_cuts, on byte offsets
            u32 a[4], c[4];
#pragma unroll
            for (u32 j = 0; j < 4; ++j) { a[j] = p4[j] + step4; c[j] = *(const u32 *)(cut_b + a[j]); }
#pragma unroll
            for (u32 j = 0; j < 4; ++j) p4[j] = c[j] <= key[j] ? a[j] : p4[j];
        }
        float cen[4];
#pragma unroll
        for (u32 j = 0; j < 4; ++j) cen[j] = *(const float *)(cen_b + p4[j]);
        // the codes (index + 1) of four consecutive values, nbits each: p4 + 4 is four times the code
        u32 field = (p4[0] + 4u) >> 2;
#pragma unroll
        for (u32 j = 1; j < 4; ++j) field |= (p4[j] + 4u) << (nbits * j - 2u);
#pragma unroll
        for (u32 j = 0; j < 4; ++j) {
            float x = v[4 * q + j];
            asm volatile("" : "+v"(x));            // widened here, not when the value arrived (thirty-two doubles would not fit)
            const double d = (double)x - (double)cen[j];
            obj += d * d;
        }
        // into the chunk's bit stream at bit (first element) * nbits: at most two 32-bit words
        const u32 bitpos = (q * EXCP_THREADS + tid) * 4u * nbits, wi = bitpos >> 5, sh = bitpos & 31u;
        atomicOr(&s_pack[wi], field << sh);
        if (sh && (field >> (32u - sh))) atomicOr(&s_pack[wi + 1], field >> (32u - sh));
        __builtin_amdgcn_sched_barrier(0);         // one group at a time: nothing of the next is started early
    }
    return obj;
}

// ---------------------------------------------------------------- final assignment + packing
// A chunk's codes are ORed, four at a time, into the chunk's bit stream in LDS and leave as whole
// 64-bit words.
__global__ __launch_bounds__(EXCP_THREADS, 5) void k_assign_pack(Workspace w, GroupParams g) {
    __shared__ float s_C[EXCP_MAX_K + 1];
    __shared__ u32 s_cut[EXCP_MAX_K + 1];
    __shared__ u32 s_pack2[2][EXCP_CHUNK * 8 / 32 + 2];  // a chunk's packed codes (up to 8 bits each); chunks alternate between the two
    __shared__ double s_red[EXCP_THREADS / 64];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 total = *w.chunk_total;
    const u32 G = gridDim.x, b = blockIdx.x;
    const u32 lo = (u32)(((u64)b * total) / G), hi = (u32)(((u64)(b + 1) * total) / G);
    if (lo >= hi) return;
    const u32 nseg = 3u * g.ntensors;
    const int K = g.K;
    u32 kp2 = 1; while (kp2 < (u32)K) kp2 <<= 1;
    const u32 nbits = (u32)g.nbits;
    const u32 words_per_chunk = EXCP_CHUNK * nbits / 64u;

    u32 sidx = 0xffffffffu, s_end = 0;
    u64 len = 0, nwords = 0;                       // of the stream in hand: fetched when the stream changes, not per chunk
    u32 chunk0 = 0;
    const EXCP_GLOBAL float *data = nullptr;
    u64 *out = nullptr;
    double obj = 0.0;                              // this thread's share of the objective over the chunks of the stream in hand
    // The workgroup's total for the stream goes into the entry of the last of its chunks (the others hold 0).
    auto close_stream = [&](u32 last_chunk) {
#pragma unroll
        for (int mm = 32; mm >= 1; mm >>= 1) obj += shfl_xor_f64(obj, mm);
        if (lane == 0) s_red[wave] = obj;
        __syncthreads();
        if (tid == 0) w.part_obj[last_chunk] = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
        obj = 0.0;
    };
    for (u32 c = lo; c < hi; ++c) {
        u32 *s_pack = s_pack2[c & 1u];
        if (sidx == 0xffffffffu || c >= s_end) {
            if (sidx != 0xffffffffu) close_stream(c - 1u);
            __syncthreads();
            sidx = find_owner(w.seg_chunk_begin, nseg, c);
            s_end = w.seg_chunk_begin[sidx + 1];
            const u32 t = sidx / 3u, which = sidx % 3u;
            const TState &T = w.st[t];
            len = w.seg[sidx].len; chunk0 = w.seg[sidx].chunk_begin; data = gptr(seg_data(w, sidx));
            nwords = excp_words(len * nbits);
            out = (u64 *)(w.desc[t].blob + (which == 0 ? T.off_cw : (which == 1 ? T.off_cm : T.off_cv)));
            for (u32 k = tid; k < (u32)K; k += EXCP_THREADS) s_C[k] = w.seg[sidx].C[k];
            __syncthreads();
            compute_cut_keys(s_C, K, s_cut);       // the final centres' cut keys
            __syncthreads();
        }
        const u64 ebase = (u64)(c - chunk0) * EXCP_CHUNK;
        const u32 clen = (len - ebase) < EXCP_CHUNK ? (u32)(len - ebase) : EXCP_CHUNK;
        const u64 wbase = (u64)(c - chunk0) * words_per_chunk;
        float v[PER_THREAD];
        load_chunk(data + ebase, clen, v);
        for (u32 i = tid; i < 2u * words_per_chunk + 2u; i += EXCP_THREADS) s_pack[i] = 0;
        __syncthreads();
        if (clen == EXCP_CHUNK) {
            obj += assign_whole_chunk(v, s_cut, s_C, kp2, nbits, s_pack);
        } else {
            // a stream's ragged last chunk: value by value
#pragma unroll
            for (u32 q = 0; q < PER_THREAD / 4; ++q) {
                u32 field = 0;
#pragma unroll
                for (u32 j = 0; j < 4; ++j) {
                    const u32 it = 4 * q + j;
                    if (chunk_elem(it) < clen) {
                        const u32 pick = centre_by_cuts(s_cut, kp2, key_of(v[it]));
                        const double d = (double)v[it] - (double)s_C[pick];
                        obj += d * d;
                        field |= (1u + pick) << (nbits * j);
                    }
                }
                const u32 bitpos = chunk_elem(4 * q) * nbits, wi = bitpos >> 5, sh = bitpos & 31u;
                if (field) {
                    atomicOr(&s_pack[wi], field << sh);
                    if (sh && (field >> (32u - sh))) atomicOr(&s_pack[wi + 1], field >> (32u - sh));
                }
            }
        }
        __syncthreads();
        for (u32 wl = tid; wl < words_per_chunk; wl += EXCP_THREADS) {
            const u64 wg = wbase + wl;
            if (wg >= nwords) break;
            out[wg] = (u64)s_pack[2 * wl] | ((u64)s_pack[2 * wl + 1] << 32);
            if (wg == nwords - 1 && (nwords & 1ull)) out[nwords] = 0ull;     // 16-byte padding
        }
        if (tid == 0) w.part_obj[c] = 0.0;
        // (no barrier here: the next chunk uses the other buffer, and this one is zeroed again only after
        // the two barriers of that chunk)
    }
    close_stream(hi - 1u);
}

// ---------------------------------------------------------------- no quantisation: the streams as they are
// Prune-only mode (Table "abl"): every survivor stream goes into its blob section as fp32, in index
// order; the section's padding (up to 16 bytes) is zeroed.  One chunk of 8192 values per step.
__global__ __launch_bounds__(EXCP_THREADS) void k_store_raw(Workspace w, GroupParams g) {
    const u32 tid = threadIdx.x;
    const u32 total = *w.chunk_total;
    const u32 nseg = 3u * g.ntensors;
    for (u32 c = blockIdx.x; c < total; c += gridDim.x) {
        const u32 sidx = find_owner(w.seg_chunk_begin, nseg, c);
        const SegState &S = w.seg[sidx];
        const u32 t = sidx / 3u, which = sidx % 3u;
        const TState &T = w.st[t];
        const u64 len = S.len;
        const u64 base = (u64)(c - S.chunk_begin) * EXCP_CHUNK;
        const u32 clen = (len - base) < EXCP_CHUNK ? (u32)(len - base) : EXCP_CHUNK;
        const u64 off = which == 0 ? T.off_cw : (which == 1 ? T.off_cm : T.off_cv);
        const EXCP_GLOBAL float *src = gptr(seg_data(w, sidx)) + base;
        EXCP_GLOBAL float *dst = gptr((float *)(w.desc[t].blob + off)) + base;
        const u32 padded = (clen + 3u) & ~3u;              // a chunk starts on a 16-byte boundary of the section
        for (u32 i = tid * 4u; i < padded; i += EXCP_THREADS * 4u) {
            f4u o;
            if (i + 4u <= clen) {
                const f4u q = *(const EXCP_GLOBAL f4u *)(src + i);
                o = q;
            } else {
                o.x = i < clen ? src[i] : 0.f; o.y = i + 1u < clen ? src[i + 1u] : 0.f;
                o.z = i + 2u < clen ? src[i + 2u] : 0.f; o.w = 0.f;
            }
            *(EXCP_GLOBAL f4u *)(dst + i) = o;
        }
    }
}

// ---------------------------------------------------------------- header, codebooks, results
__global__ __launch_bounds__(EXCP_THREADS) void k_finalize(Workspace w, GroupParams g, u32 rec_base) {
    __shared__ double s_obj[3];
    const u32 t = blockIdx.x, tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const TDesc &D = w.desc[t];
    TState &T = w.st[t];
    const bool raw = (u32)g.nbits >= EXCP_RAW_BITS;          // no quantisation: no codebooks, no objective
    const u32 E = raw ? 0u : 1u << g.nbits;
    if (wave < 3) {
        const u32 sidx = 3u * t + wave;
        double acc = 0.0;
        if (!raw && w.seg[sidx].len) {
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
        case 1: hipLaunchKernelGGL(k_km_clear_counts, dim3(excp_grid(w, 8)), dim3(EXCP_THREADS), 0, s, w, g); break;
        case 2:
            hipLaunchKernelGGL(k_km_scan_parts, dim3(nseg * SCAN_PARTS), dim3(1024), 0, s, w, g);
            hipLaunchKernelGGL(k_km_scan, dim3(nseg), dim3(NBKT), 0, s, w, g);
            hipLaunchKernelGGL(k_km_scan_apply, dim3(nseg * SCAN_PARTS), dim3(1024), 0, s, w, g);
            break;
        case 3: hipLaunchKernelGGL(k_km_scatter, dim3(excp_grid(w, 1)), dim3(SC_THREADS), 0, s, w, g); break;
        case 4:
            if (g.wide == 2u) hipLaunchKernelGGL((k_km_bucket_stats<16, 1>), dim3(nseg * NBKT), dim3(1024), 0, s, w, g);
            else if (g.wide) hipLaunchKernelGGL((k_km_bucket_stats<16, 4>), dim3(nseg * (NBKT / 4)), dim3(1024), 0, s, w, g);
            else hipLaunchKernelGGL((k_km_bucket_stats<4, 4>), dim3(std::min(nseg * (NBKT / 4), excp_grid(w, 32))), dim3(256), 0, s, w, g);
            break;
        default: break;
    }
}

void launch_km_init(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    if (g.wide) hipLaunchKernelGGL(k_km_init<1024>, dim3(3 * g.ntensors * (u32)g.K), dim3(1024), 0, s, w, g);
    else hipLaunchKernelGGL(k_km_init<256>, dim3(3 * g.ntensors * (u32)g.K), dim3(256), 0, s, w, g);
}

void launch_km_classify(const Workspace &w, const GroupParams &g, int iteration, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_km_classify, dim3(3 * g.ntensors), dim3(EXCP_THREADS), 0, s, w, g,
                       (u32)(iteration & 1), (u32)(iteration > 0));
}

void launch_km_iter(const Workspace &w, const GroupParams &g, int iteration, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_km_iter, dim3(excp_grid(w, 20)), dim3(EXCP_THREADS), 0, s, w, g, (u32)(iteration & 1));
}

void launch_km_update(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_km_update, dim3(3 * g.ntensors), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_assign_pack(const Workspace &w, const GroupParams &g, hipStream_t s) {
    hipLaunchKernelGGL(k_assign_pack, dim3(excp_grid(w, 5)), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_store_raw(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_store_raw, dim3(excp_grid(w, 16)), dim3(EXCP_THREADS), 0, s, w, g);
}

void launch_finalize(const Workspace &w, const GroupParams &g, hipStream_t s) {
    if (!g.ntensors) return;
    hipLaunchKernelGGL(k_finalize, dim3(g.ntensors), dim3(EXCP_THREADS), 0, s, w, g, w.rec_base);
}
