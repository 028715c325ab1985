// Small device helpers shared by the ExCP kernels (wave64, gfx950).
#pragma once
#include "excp_device.h"

#define WAVE 64

__device__ __forceinline__ u32 f2u(float x) { return __float_as_uint(x); }
__device__ __forceinline__ float u2f(u32 x) { return __uint_as_float(x); }

__device__ __forceinline__ u64 ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }
__device__ __forceinline__ u32 lane_id() { return threadIdx.x & 63u; }
// number of set bits of a wave-wide mask that belong to lanes below the calling one
__device__ __forceinline__ u32 lanes_below(unsigned long long m) {
    return __builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, 0u));
}
__device__ __forceinline__ u64 lanemask_lt() { return (1ull << lane_id()) - 1ull; }

__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int m) {
    u32 lo = (u32)v, hi = (u32)(v >> 32);
    lo = __shfl_xor(lo, m, WAVE);
    hi = __shfl_xor(hi, m, WAVE);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 wave_sum_u64(u64 v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += shfl_xor_u64(v, m);
    return v;
}
__device__ __forceinline__ u32 wave_sum_u32(u32 v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, WAVE);
    return v;
}
__device__ __forceinline__ u32 wave_max_u32(u32 v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = max(v, (u32)__shfl_xor(v, m, WAVE));
    return v;
}
__device__ __forceinline__ double shfl_xor_f64(double v, int m) {
    return __longlong_as_double((long long)shfl_xor_u64((u64)__double_as_longlong(v), m));
}

// Histogram increment in LDS for data that may be heavily tied (then most lanes of a wave hit the same
// bin, and plain atomics take turns): up to two groups of lanes that share a bin are added by one lane
// each, whoever is left adds for itself.  Every lane of the wave must call it.
__device__ __forceinline__ void hist_add_tied(u32 *hist, u32 bin, bool active) {
    u64 todo = ballot64(active);
#pragma unroll
    for (int round = 0; round < 2; ++round) {
        if (todo == 0ull) break;                            // the same in every lane
        const u32 leader = (u32)__ffsll((long long)todo) - 1u;
        const u32 lb = (u32)__shfl((int)bin, (int)leader, WAVE);
        const u64 same = ballot64(active && bin == lb) & todo;
        if (lane_id() == leader) atomicAdd(&hist[lb], (u32)__popcll(same));
        todo &= ~same;
    }
    if ((todo >> lane_id()) & 1ull) atomicAdd(&hist[bin], 1u);
}

// Largest t with begin[t] <= x (begin is non-decreasing, begin[0] == 0, count+1 entries,
// begin[count] > x).  Entries may repeat (empty items); the item found is never empty.
__device__ __forceinline__ u32 find_owner(const u32 *__restrict__ begin, u32 count, u32 x) {
    u32 lo = 0, hi = count;          // invariant: begin[lo] <= x < begin[hi]
    while (hi - lo > 1) {
        u32 mid = (lo + hi) >> 1;
        if (begin[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// Pointers read from descriptor tables are generic to the compiler; these casts state that they
// point to global memory, which turns flat loads/stores into global ones with immediate offsets.
#define EXCP_GLOBAL __attribute__((address_space(1)))
#define EXCP_CONSTANT __attribute__((address_space(4)))      // global memory that the kernel at hand only reads
template <class T>
__device__ __forceinline__ const EXCP_GLOBAL T *gptr(const T *p) { return (const EXCP_GLOBAL T *)(uintptr_t)p; }
template <class T>
__device__ __forceinline__ EXCP_GLOBAL T *gptr(T *p) { return (EXCP_GLOBAL T *)(uintptr_t)p; }

// Weights stored in 16 bits (flags bits 4-5 of a compress call or a blob header: 1 = IEEE binary16,
// 2 = bfloat16).  Widening is exact; narrowing rounds to nearest even (a finite fp32 beyond the
// format's range becomes infinity, as IEEE conversion does).  All arithmetic stays fp32.
__device__ __forceinline__ u32 excp_wtype(u32 flags) { return (flags >> 4) & 3u; }
__device__ __forceinline__ float w16_widen(u32 h, bool bf) {
    const float half = (float)__builtin_bit_cast(_Float16, (unsigned short)h);
    return bf ? u2f(h << 16) : half;
}
__device__ __forceinline__ u32 w16_narrow(float x, bool bf) {
    const u32 b = f2u(x);
    const u32 bf_bits = (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;       // never a NaN here: inputs are finite
    const u32 half_bits = (u32)__builtin_bit_cast(unsigned short, (_Float16)x);
    return bf ? bf_bits : half_bits;
}
typedef unsigned short us4 __attribute__((ext_vector_type(4), aligned(8)));
// One weight at index idx of an array whose element type is given by wt (0 = fp32).
__device__ __forceinline__ float load_weight(const float *p, u64 idx, u32 wt) {
    if (wt == 0u) return p[idx];
    return w16_widen(((const unsigned short *)p)[idx], wt == 2u);
}
__device__ __forceinline__ void store_weight(float *p, u64 idx, u32 wt, float x) {
    if (wt == 0u) p[idx] = x;
    else ((unsigned short *)p)[idx] = (unsigned short)w16_narrow(x, wt == 2u);
}

// Four consecutive weights of a tile: elements [off, off + 4) of the tile that starts at `tile0` (an
// element pointer into an array of type wt), of which `rem` exist; one 16-byte (fp32) or 8-byte
// (16-bit, if the array is 8-byte aligned) load where all four exist, else one by one; missing ones are 0.
typedef float f4w __attribute__((ext_vector_type(4), aligned(4)));
__device__ __forceinline__ void load_weights4(const float *arr, u64 tile0, u32 off, u32 rem, u32 wt, float (&out)[4]) {
    if (off + 4u <= rem && wt == 0u) {
        const f4w q = *(const EXCP_GLOBAL f4w *)(gptr(arr) + tile0 + off);
        out[0] = q.x; out[1] = q.y; out[2] = q.z; out[3] = q.w;
    } else if (off + 4u <= rem && ((uintptr_t)arr & 7u) == 0u) {
        const us4 q = *(const EXCP_GLOBAL us4 *)(gptr((const unsigned short *)arr) + tile0 + off);
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = w16_widen(q[j], wt == 2u);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = (off + (u32)j < rem) ? load_weight(arr, tile0 + off + (u32)j, wt) : 0.f;
    }
}

// Copy of a tile table in LDS (the per-tile owner search then costs no global round trips).
#define EXCP_MAX_GROUP_TENSORS 1024
__device__ __forceinline__ void load_tile_table(u32 *dst, const u32 *__restrict__ src, u32 count) {
    for (u32 i = threadIdx.x; i <= count; i += blockDim.x) dst[i] = src[i];
    __syncthreads();
}

// ---- value -> bucket map of the codebook stage (built by k_km_sample)
constexpr u32 HALF_CELLS = EXCP_KM_CELLS / 2;

// Value -> cell, monotone in the value: negative values fill cells 2047 down to 0 as their
// magnitude grows, positive ones 2048 up to 4095.  map[0..3] = offset and shift of the negative
// side, offset and shift of the positive side; magnitudes beyond the sampled range clamp.
__device__ __forceinline__ u32 cell_of(float x, const u32 *map) {
    const u32 bits = f2u(x), a = bits & 0x7fffffffu;
    const bool neg = bits >> 31;
    const u32 amin = neg ? map[0] : map[2], sh = neg ? map[1] : map[3];
    const u32 c = min((max(a, amin) - amin) >> sh, HALF_CELLS - 1u);
    return neg ? (c ^ (HALF_CELLS - 1u)) : (c | HALF_CELLS);
}
__device__ __forceinline__ u32 bucket_of(float x, const u32 *map) {
    return ((const unsigned char *)(map + 4))[cell_of(x, map)];
}

// Order-preserving map of fp32 bit patterns to unsigned keys (and back).
__device__ __forceinline__ u32 key_of(float x) {
    u32 u = f2u(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float val_of(u32 k) {
    return u2f((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Index of the nearest centre of x among centres in ascending order (Sec. 3.3 leaves the rule
// open; this is the rule the library fixes).  a = last centre <= x, b = the next one; the two
// distances are evaluated in fp64 with one rounding each, b wins only if strictly nearer, and
// among centres of equal value the lowest index is taken.  dist_out receives (x - C[pick])^2.
__device__ __forceinline__ int nearest_centre(float x, const float *C, int K, double *dist_out) {
    int lo = 0, hi = K;                    // count of centres <= x by bisection
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (C[mid] <= x) lo = mid + 1; else hi = mid;
    }
    int j = lo - 1;                        // largest index with C[j] <= x, or -1
    int a = j < 0 ? 0 : j;
    int b = (j + 1 < K) ? j + 1 : K - 1;
    double xd = (double)x;
    double da = fabs(xd - (double)C[a]);
    double db = fabs((double)C[b] - xd);
    int pick = (db < da) ? b : a;
    float cv = C[pick];
    while (pick > 0 && C[pick - 1] == cv) --pick;
    if (dist_out) { double d = xd - (double)cv; *dist_out = d * d; }
    return pick;
}

// The nearest-centre rule is monotone in the value, so it is fully described by K - 1 cut keys:
// cut[k] = smallest key (order-preserving bit pattern) of a finite value whose nearest centre has
// index >= k, or 0xffffffff when no finite value reaches k.  Found by bisection with the rule
// itself, so "number of cut keys <= key(x)" IS nearest_centre(x), bit for bit.  Threads 1..K-1 of
// the workgroup each find one; entries from K up to 255 are set to 0xffffffff.  C and cut are LDS
// arrays of 256 entries; the caller synchronises before and after.
__device__ __forceinline__ void compute_cut_keys(const float *C, int K, u32 *cut) {
    const u32 k = threadIdx.x;
    if (k == 0 || k > 255u) return;
    u32 res = 0xffffffffu;
    if ((int)k < K) {
        constexpr u32 KEY_LO = 0x00800000u, KEY_HI = 0xff7fffffu;          // keys of -FLT_MAX and +FLT_MAX
        auto reaches = [&](u32 key) { return (u32)nearest_centre(val_of(key), C, K, nullptr) >= k; };
        // The border between centres k-1 and k lies next to their midpoint, so a bracket of a few keys
        // around the midpoint is probed first; whatever the probes say, the bisection below starts
        // from a bracket they have proved (every key below lo stays below k, hi reaches k), so the
        // result is that of a bisection over all finite keys.
        const u32 mk = key_of((float)(0.5 * ((double)C[k - 1] + (double)C[k])));
        const u32 p_lo = mk - KEY_LO > 2u ? mk - 2u : KEY_LO, p_hi = KEY_HI - mk > 2u ? mk + 2u : KEY_HI;
        u32 lo = KEY_LO, hi = KEY_HI;
        bool any = true;
        if (reaches(p_hi)) {
            if (reaches(p_lo)) hi = p_lo; else { lo = p_lo + 1u; hi = p_hi; }
        } else if (p_hi < KEY_HI && reaches(KEY_HI)) {
            lo = p_hi + 1u;
        } else {
            any = false;                                                   // no finite value reaches k
        }
        if (any) {
            while (lo < hi) {                                              // invariant: hi reaches k
                const u32 mid = lo + ((hi - lo) >> 1);
                if (reaches(mid)) hi = mid; else lo = mid + 1u;
            }
            res = hi;
        }
    }
    cut[k] = res;
}

// Number of cut keys <= key, i.e. the index of the nearest centre.  kp2 = smallest power of two >= K.
__device__ __forceinline__ u32 centre_by_cuts(const u32 *cut, u32 kp2, u32 key) {
    u32 lo = 0;
    for (u32 step = kp2 >> 1; step >= 1; step >>= 1)
        if (cut[lo + step] <= key) lo += step;
    return lo;
}
