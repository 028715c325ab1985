// Device-side tables shared by the ExCP kernels and their host orchestrator.
// One "group" of tensors is processed by every kernel at once: kernels walk a
// tile list (EXCP_TILE elements per tile, tiles of all tensors back to back)
// or a chunk list (EXCP_CHUNK survivors per chunk) and find their tensor from
// these tables, so no launch depends on a value that only the device knows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define EXCP_TILE        4096u     // elements per tile of the full-tensor passes (256 threads x 16)
#define EXCP_CHUNK       8192u     // survivors per chunk of the survivor passes
#define EXCP_SUPER_CHUNKS 16u      // chunks per unit of the bucket counts (and of the scatter's workgroup ranges)
#define EXCP_THREADS     256
#define EXCP_ABSM_BINS   40        // u64 accumulators, 8 binary exponents apart, for the exact sum of |m|
#define EXCP_MAX_K       255
#define EXCP_KM_CELLS    4096u     // cells of the value -> bucket map (2048 per sign)
#define EXCP_KM_MAP_WORDS (4u + EXCP_KM_CELLS / 4u)
#define EXCP_HEADER      80u
#define EXCP_MAGIC       0x50435845u
#define EXCP_VERSION     1u

typedef unsigned long long u64;
typedef unsigned int u32;

// Host-filled description of one tensor of a compress group.
struct TDesc {
    const float *Wp, *W, *m, *v;
    u64 n;
    unsigned char *blob;
    u64 blob_cap;
    float *W_out;
    u64 elem_off;      // start of this tensor's survivor slots in the group workspace
    u64 cand_off;      // start and capacity of this tensor's median-candidate list
    u64 cand_cap;
    u32 cand_lists;    // the candidate list of a very large tensor is cut into this many lists (1 .. 16), each with a
    u32 pad0;          // counter of its own, so that thousands of waves do not queue at one address
    u32 tile_begin;    // first tile of this tensor in the group's tile list
    u32 tile_count;
};

// Device-written per-tensor state of a compress group.
struct TState {
    u64 absm[EXCP_ABSM_BINS];   // sum_g absm[g] * 2^(8g - 149) == exact sum of |m|
    u64 nonfinite;
    u64 n_w, n_o;
    u64 off_bo, off_cw, off_cm, off_cv, blob_bytes;
    double abs_sum;
    double obj[3];
    u32 br_lo, br_hi;           // median bracket (keys) from the sorted sample
    u32 med_state;              // 0 select among candidates pending, 1 median known, 2 full-tensor fallback
    u32 cand_count, cand_overflow, c_lt;   // keys inside / overflowing the list / below the bracket
    u32 sel_base, sel_width;    // radix select: key bits decided so far, number of undecided low bits
    u32 sel_rank;               // rank still to find among the undecided keys
    u32 med_bits;
    float mean32, t_w, r_o;
    int status;
    u32 absm_base;              // lowest bit position of the 24-position window used for the exact sum of |m|
    // tied data (16-bit weights): values inside the median bracket that the sample shows to be heavily
    // repeated are counted, not listed among the candidates
    u32 natoms, atom_key[4], atom_cnt[4];
    u32 pad2[2];
};

// One survivor stream (3 per tensor: residual, m, v) during codebook construction.
struct SegState {
    u64 len;
    u32 chunk_begin;            // first chunk of this stream in the group's chunk list
    u32 pad;
    float C[EXCP_MAX_K + 1];    // current centres (K used)
    u32 cut[EXCP_MAX_K + 1];    // cut[k], 1 <= k < K: smallest key whose nearest centre has index >= k
};

// Host-filled description of one tensor of a decompress group.
struct DDesc {
    const float *Wp;
    const unsigned char *blob;
    u64 blob_bytes;
    u64 n;
    float *W_out, *m_out, *v_out;
    // per-element code tensors (two codes of 4 bits or fewer per byte, else one per byte): written by
    // the export of a blob, read by the reconstruction from that layout (then `blob` is the header
    // with the codebooks and `head` is unused)
    unsigned char *cw, *cm, *cv;
    unsigned char *head;        // export: receives header and codebooks (nullable)
    u32 tile_begin, tile_count;
    u32 wtype;                  // storage of the caller's weight arrays (0 fp32, 1 fp16, 2 bf16): the blob must
    u32 pad;                    // say the same; 3 = no weight arrays are involved
};

struct DState {
    u64 n_w, n_o, blob_bytes;
    u64 off_bw, off_bo, off_cw, off_cm, off_cv;
    u32 nbits;
    int status;
    u64 pop_w, pop_o;           // bitmap populations found while scanning
    u32 flags;                  // the blob's flags (bit 3: bitmap_o covers all elements)
    u32 pad;
};

// Host-filled description of one tensor of a chain reconstruction: its decode descriptors (one per
// compressed checkpoint, oldest first) are ddesc[first_desc .. first_desc + steps).
struct CDesc {
    const float *W0;
    float *W_out;
    u64 n;
    u32 first_desc, steps;
    u32 tile_begin, tile_count;     // in the group's list of tensor tiles
};

// Result record copied back to the host after a batch.
struct HostRec {
    u64 n, n_w, n_o, blob_bytes, nonfinite;
    double abs_sum, obj[3];
    float med, mean32, t_w, r_o;
    int status;
    int pad;
};

struct GroupParams {
    float alpha, beta;
    int nbits, K, iters;
    u32 flags;
    u32 ntensors, ntiles;
    u32 wide;                   // per-bucket kernels with sixteen waves: 1 = tied data (16-bit weights), 2 = a very large
                                // tensor in the group (then also one bucket per workgroup)
};

#define EXCP_RAW_BITS    32u       // "code" width of a blob written without quantisation: fp32 values, no codebooks
// bytes of the three codebooks that follow the header
static __host__ __device__ inline u64 excp_books_bytes(u32 nbits) { return nbits >= EXCP_RAW_BITS ? 0ull : 12ull << nbits; }
static __host__ __device__ inline u64 excp_pad16(u64 b) { return (b + 15ull) & ~15ull; }
static __host__ __device__ inline u64 excp_words(u64 bits) { return (bits + 63ull) >> 6; }

// ---- launchers (defined next to their kernels) --------------------------------------------
struct Workspace {
    // group tables
    TDesc *desc; TState *st; SegState *seg; u32 *tile_begin;   // tile_begin has ntensors+1 entries
    // survivors
    float *xw, *xm, *xv;
    // median select
    u32 *med_hist;            // [tensor][2048]
    u32 *cand;                // median candidates (keys inside the sample bracket), per tensor
    u32 *cand_ctr;            // [tensor][16][32] per list: [0] slots asked for, [1] end of the slots granted (128 B apart)
    // mask pass
    u64 *tile_status;         // per 2048-element sub-tile: survivors << 32 | moment survivors
    u64 *mask_prefix;         // exclusive scan of tile_status within each tensor
    u64 *mask_part;           // [tensor][16] packed counts of each sixteenth of a tensor's sub-tiles
    u64 *mask_bo;             // [sub-tile][32] M_o bits of the sub-tile's survivors, local positions
    // survivor passes
    u32 *chunk_total;         // [1]
    u32 *seg_chunk_begin;     // [segments + 1] first chunk of every survivor stream
    float *pw, *pm, *pv;      // survivors partitioned into value-ordered buckets (same offsets as xw/xm/xv)
    u32 *km_split;            // [segment][EXCP_KM_MAP_WORDS] value -> bucket map: 4 parameters, then 4096 bucket bytes
    u32 *km_cnt;              // [chunk][256] bucket counts, then positions, of every chunk
    u32 *km_begin;            // [segment][257] first position of every bucket
    u32 *km_part;             // [segment][16][256] bucket counts, then first positions, of each sixteenth of a stream's chunks
    u64 *km_bsum;             // [segment][256][EXCP_ABSM_BINS] exact signed sum of every bucket
    u32 *km_min, *km_max;     // [segment][256] smallest / largest key of every bucket
    u64 *km_acc;              // [segment][EXCP_MAX_K][EXCP_ABSM_BINS + 1] per-centre exact sum and count
    void *km_items;           // work items of the Lloyd accumulation (cut buckets in pieces)
    u32 *km_item_count;       // [2] lengths of the two work lists used by alternate iterations
    u32 km_item_cap;
    double *part_obj;         // [chunk]
    u32 max_chunks;
    // decode
    DDesc *ddesc; DState *dst;
    CDesc *cdesc; u32 *chain_tile_begin;   // chain reconstruction: tensors and their tile table
    u32 *dec_cnt_w, *dec_cnt_o;   // per tile counts -> exclusive bases
    u64 *dec_part;                // [descriptor][16] tile-count totals of each sixteenth of a tensor's tiles
    u32 *dec_kinds;               // [1] kinds of blob in the group being decoded: 1 fp32 weights, 2 16-bit weights, 4 unquantised
    // flags
    int *err_flag;
    HostRec *rec_dev;
    u32 rec_base;             // index of this group's first tensor in rec_dev
    int cus;                  // compute units of the device
};

// Grid of a persistent kernel: `per_cu` workgroups per compute unit (each kernel's figure was
// measured on its own).
static inline u32 excp_grid(const Workspace &w, u32 per_cu) { return (u32)w.cus * per_cu; }

void launch_zero_u32(u32 *p, u64 count, hipStream_t s);
void launch_copy_probe(const void *src, void *dst, u64 bytes, hipStream_t s);
void launch_stats(const Workspace &w, const GroupParams &g, int phase, hipStream_t s);
void launch_mask_compact(const Workspace &w, const GroupParams &g, int phase, hipStream_t s);
void launch_layout(const Workspace &w, const GroupParams &g, hipStream_t s);
void launch_km_partition(const Workspace &w, const GroupParams &g, int phase, hipStream_t s);
void launch_km_init(const Workspace &w, const GroupParams &g, hipStream_t s);
void launch_km_classify(const Workspace &w, const GroupParams &g, int iteration, hipStream_t s);
void launch_km_iter(const Workspace &w, const GroupParams &g, int iteration, hipStream_t s);
void launch_km_update(const Workspace &w, const GroupParams &g, hipStream_t s);
void launch_assign_pack(const Workspace &w, const GroupParams &g, hipStream_t s);
void launch_finalize(const Workspace &w, const GroupParams &g, hipStream_t s);
void launch_decode_from_compress(const Workspace &w, const GroupParams &g, hipStream_t s);
void launch_decode_parse(const Workspace &w, u32 ntensors, bool allow_raw, hipStream_t s);
void launch_decode_single_setup(const Workspace &w, const DDesc &d, hipStream_t s);
void launch_decode_main16(const Workspace &w, u32 ntensors, u32 ntiles, bool moments, hipStream_t s);
void launch_decode_raw(const Workspace &w, u32 ntensors, u32 ntiles, bool moments, hipStream_t s);
void launch_store_raw(const Workspace &w, const GroupParams &g, hipStream_t s);
void launch_decode_count(const Workspace &w, u32 ntensors, u32 ntiles, int which, hipStream_t s);
void launch_decode_scan(const Workspace &w, u32 ntensors, int which, hipStream_t s);
void launch_decode_main(const Workspace &w, u32 ntensors, u32 ntiles, bool moments, hipStream_t s);
void launch_decode_finish(const Workspace &w, u32 ntensors, hipStream_t s);
void launch_export_dense(const Workspace &w, u32 ntensors, u32 ntiles, bool moments, hipStream_t s);
void launch_dense_parse(const Workspace &w, u32 ntensors, hipStream_t s);
void launch_decode_dense(const Workspace &w, u32 ntensors, u32 ntiles, hipStream_t s);
void launch_decode_chain(const Workspace &w, u32 ntensors, u32 ntiles, hipStream_t s);
void launch_chain_finish(const Workspace &w, u32 ntensors, hipStream_t s);
