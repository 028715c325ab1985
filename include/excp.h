/*
 * excp.h -- C ABI of the MI355X (gfx950) ExCP checkpoint-compression hot path.
 *
 * What is computed (per flat fp32 tensor; "ExCP", arxiv 2406.11257):
 *   compress   = Alg. 1 without its last, general-purpose archive step:
 *                residual against the previous *reconstructed* weights
 *                (Sec. 3.1, Eq. "ckpt_res"), joint weight / momentum pruning
 *                (Sec. 3.2, Eq. "r_w" and Eq. "r_o"), k-means codebook
 *                quantisation of the survivors to 2^nbits - 1 centres with code
 *                0 kept for "pruned" (Sec. 3.3, Sec. 4.2), bit packing
 *                (Sec. 4.2) -- plus the reconstructed weights that Sec. 3.4
 *                says are kept for the next step.
 *   decompress = Alg. 2: codebook look-up and add to the previous weights.
 *
 * Naming.  The paper swaps the usual Adam symbols.  Here `m` is the FIRST
 * moment (signed), `v` the SECOND moment (non-negative, under the square root
 * of Eq. "r_w").
 *
 * Exact definition (all fp32 operations are IEEE binary32, round to nearest
 * even, one rounding each, no fused multiply-add, denormals kept):
 *   d_i    = W_t[i] - W_prev_recon[i]
 *   med    = the ((n-1)/2)-th smallest of |d_i|  (0-based; lower median)
 *   t_w    = alpha * med ;  r_i = t_w / sqrt(v_i) ;  M_w(i) = |d_i| > r_i
 *   mean   = fp32( fp64(exact sum of |m_i|) / n ) ; r_o = beta * mean
 *   M_o(i) = M_w(i) and |m_i| > r_o
 *   streams: d at M_w (n_w values), m and v at M_o (n_o values each), in
 *   index order; each stream is clustered on its own: K = 2^nbits - 1 centres
 *   start at the order statistics of rank ((2k+1) len)/(2K), then exactly
 *   `lloyd_iters` updates (nearest centre: of the two centres that bracket a
 *   value the upper one wins only if its fp64 distance is strictly smaller, and
 *   of equal centres the lowest index is taken; centre = fp32(exact sum rounded
 *   once to fp64 / count); empty clusters keep their centre; the centres are
 *   re-sorted ascending after every update, which only matters for heavily tied
 *   data); code = 1 + index of the nearest final centre.
 *   reconstruct: W_hat[i] = W_prev_recon[i] + C_w[code] at M_w, else
 *   W_prev_recon[i]; m_hat, v_hat = C[code] at M_o, else +0.
 *
 * The other modes of the paper's ablation tables need no switch: without the residual (Table "abl")
 * pass zeros as W_prev_recon; without pruning pass alpha = beta = 0 (only exact zeros are dropped).
 *
 * Compressed tensor ("blob"), little endian, every section padded to 16 B:
 *   header (80 B): u32 magic "EXCP", u32 version=1, u32 nbits, u32 flags,
 *                  u64 n, u64 n_w, u64 n_o, f32 alpha, beta, med, mean, t_w,
 *                  r_o, u64 blob_bytes, u32 lloyd_iters, u32 0
 *   3 codebooks  : 2^nbits fp32 each (weights, m, v); entry 0 = +0.0
 *   bitmap_w     : ceil(n/64)   u64, bit (i & 63) of word (i >> 6) = M_w(i)
 *   bitmap_o     : ceil(n_w/64) u64 over the M_w survivors in index order (with EXCP_FLAG_NO_W2M:
 *                  ceil(n/64) u64 over all elements)
 *   codes_w/m/v  : nbits-wide codes, element j in bits [j*nbits, (j+1)*nbits)
 *                  of a little-endian bit stream stored as u64 words
 *
 * Memory and ownership.  Every tensor pointer below is DEVICE memory on the
 * context's GPU (4-byte aligned is enough; weights are fp32 unless EXCP_FLAG_W_* says otherwise); blobs are DEVICE memory, 16-byte
 * aligned.  The caller owns all of them and the HIP stream.  The context owns
 * only its workspace and its bookkeeping lists, allocated in excp_create; the
 * compress, decompress, export, chain and collect calls allocate nothing, on the
 * device or on the host (the one later allocation is the event pool that the
 * first excp_set_profiling(ctx, 1) creates, outside any step).  stats /
 * blob_bytes outputs are HOST memory.
 *
 * Execution.  Work is enqueued on the context's stream.  excp_compress_tensors
 * and excp_decompress_tensors return after enqueueing; excp_collect waits for
 * the stream and reports per-tensor results and data-dependent errors.  The
 * single-tensor calls wait themselves.  A context is not thread-safe, and a
 * new batch may be submitted only after the previous one was collected.
 *
 * Errors.  0 on success, a negative EXCP_E_* otherwise; nothing throws.
 * Argument errors are returned at once and enqueue nothing.  Data-dependent
 * errors (non-finite input, blob capacity, damaged blob) are returned by
 * excp_collect; the outputs of a failed tensor are unspecified but no memory
 * outside the caller's buffers is touched.
 */
#ifndef EXCP_H
#define EXCP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EXCP_OK            0
#define EXCP_E_ARG        -1   /* null pointer, nbits outside [2,8], negative / non-finite alpha or beta,
                                  lloyd_iters < 0, unknown flags, tensor larger than the context allows */
#define EXCP_E_CAP        -2   /* blob_cap smaller than the compressed tensor */
#define EXCP_E_NONFINITE  -3   /* NaN or Inf in an input, or the residual overflows fp32 */
#define EXCP_E_BLOB       -4   /* decompress: bad magic / version / sizes / bitmap population, a blob of another
                                  weight storage than the arrays passed, or of a kind the call does not read */
#define EXCP_E_HIP        -5   /* a HIP call failed, or the device could not be used.  If it happens while a batch
                                  is being enqueued, the call waits for what it had enqueued, and the context
                                  refuses further work with this code: destroy it */
#define EXCP_E_STATE      -6   /* call order violated (batch pending / nothing to collect) */
#define EXCP_E_INTERNAL   -7   /* an internal work list overflowed (should not happen) */

/* flags of the compress calls (stored in the blob header, which is where the readers take them from;
 * only the storage of the weight arrays is stated again by whoever reads a blob, see excp_blob) */
#define EXCP_FLAG_MEDIAN_OF_WEIGHTS 1u  /* med = lower median of |W_t| instead of |d| (the other reading of Eq. "r_w") */
#define EXCP_FLAG_NO_M2W            2u  /* ablation of Table "vit": r_i = alpha * med for every i (no 1/sqrt(v_i))   */
#define EXCP_FLAG_NO_QUANT          4u  /* Table "abl", prune without quantisation: the survivors are stored as the
                                           fp32 values they are.  nbits and lloyd_iters are ignored; the header says
                                           nbits = 32, the codebook section is empty, the three code sections hold
                                           fp32 bit patterns (32-bit "codes" in the same bit order); reconstruction
                                           adds the residual itself.  Size and bound: pass nbits = 32 below.
                                           Such blobs are read by excp_decompress_tensors only (no chain, no export). */
#define EXCP_FLAG_NO_W2M            8u  /* ablation of Table "vit", no weights-to-momentum check: M_o(i) = |m_i| > r_o
                                           whether or not the weight is kept.  bitmap_o then has one bit per ELEMENT
                                           (ceil(n/64) words) and n_o may exceed n_w; everything else is unchanged. */

#define EXCP_FLAG_W_F16             16u /* the WEIGHT arrays (W_prev_recon, W_t, W_recon_out; W0 / W_out of a chain)   */
#define EXCP_FLAG_W_BF16            32u /* hold IEEE binary16 / bfloat16 instead of fp32 (Sec. 4.3: checkpoints saved
                                           in 16 bits); at most one of the two.  2-byte aligned is enough (8-byte
                                           aligned arrays are read and written in wider pieces).  A weight is widened
                                           exactly, all arithmetic is the fp32 arithmetic above, and a reconstructed
                                           weight is the fp32 sum rounded to nearest even into the storage format;
                                           pruned positions keep their bits.  The moments stay fp32.  The header
                                           records the storage; a reader passes arrays of that storage and says
                                           so (excp_blob.flags), and a mismatch is EXCP_E_BLOB. */

#define EXCP_MAX_TENSOR_ELEMS 2147479552ull   /* per-tensor element limit (2^31 - 4096) */

typedef struct excp_ctx excp_ctx;

/* One tensor of a compress batch (Alg. 1 inputs). */
typedef struct {
    const void  *W_prev_recon;   /* device, n weights: reconstructed weights of the previous checkpoint */
    const void  *W_t;            /* device, n weights: current weights                            */
    const float *m_t;            /* device, n: Adam first moment                                  */
    const float *v_t;            /* device, n: Adam second moment                                 */
    uint64_t     n;              /* elements; 0 is allowed (header-only blob)                     */
    void        *blob;           /* device, 16-B aligned: receives the compressed tensor          */
    uint64_t     blob_cap;       /* bytes available at blob (excp_blob_bound never fails)         */
    void        *W_recon_out;    /* device, n weights, nullable: reconstructed weights of THIS
                                    checkpoint; may be the same pointer as W_prev_recon (in place) */
} excp_tensor;

/* One tensor of a decompress batch (Alg. 2 inputs). */
typedef struct {
    const void  *W_prev_recon;   /* device, n weights in the storage the blob's header names */
    const void  *blob;           /* device, 16-B aligned */
    uint64_t     blob_bytes;     /* bytes readable at blob */
    uint64_t     n;              /* must equal the n stored in the blob */
    void        *W_recon_out;    /* device, n weights, nullable; may equal W_prev_recon */
    float       *m_out;          /* device, n, nullable */
    float       *v_out;          /* device, n, nullable */
    uint32_t     flags;          /* storage of the weight arrays passed here: 0 (fp32), EXCP_FLAG_W_F16 or
                                    EXCP_FLAG_W_BF16.  Must be what the blob's header says (EXCP_E_BLOB
                                    otherwise), so that no array is ever read with the wrong element size. */
    uint32_t     reserved;       /* 0 */
} excp_blob;

/* One tensor of a chain reconstruction (Alg. 3): the weights the chain starts from and `steps`
 * compressed checkpoints, oldest first; each was compressed against the reconstruction of the one
 * before it.  `blobs` and `blob_bytes` are HOST arrays of `steps` entries; the blobs themselves are
 * device memory, 16-B aligned. */
#define EXCP_MAX_CHAIN 16
typedef struct {
    const void        *W0;          /* device, n weights: seed-initialised (or fully stored)      */
    uint64_t           n;
    int                steps;       /* 1 .. EXCP_MAX_CHAIN; longer chains: call again from W_out  */
    const void *const *blobs;       /* host array of device pointers                              */
    const uint64_t    *blob_bytes;  /* host array: bytes readable at each blob                    */
    void              *W_out;       /* device, n weights, nullable; may equal W0                  */
    float             *m_out;       /* device, n, nullable: moments stored in the LAST checkpoint */
    float             *v_out;
    uint32_t           flags;       /* storage of W0 / W_out, as in excp_blob; every checkpoint of the
                                       chain must have been written with the same storage            */
    uint32_t           reserved;    /* 0 */
} excp_chain;

/* Per-tensor results (host). */
typedef struct {
    uint64_t n, n_w, n_o;        /* elements, kept residuals, kept moment pairs        */
    uint64_t blob_bytes;         /* size of the compressed tensor                      */
    uint64_t nonfinite;          /* count of non-finite inputs seen                    */
    double   abs_sum_m;          /* exact sum of |m|, rounded once to fp64            */
    double   obj_w, obj_m, obj_v;/* final k-means objective of each stream            */
    float    median_abs_dw;      /* med                                                */
    float    mean_abs_m;         /* mean                                               */
    float    t_w, r_o;           /* alpha*med, beta*mean                               */
    int32_t  status;             /* EXCP_OK or the EXCP_E_* of this tensor             */
    int32_t  reserved;
} excp_stats;

/* Create a context on `hip_device`, working on `hip_stream` (a hipStream_t, borrowed; NULL = the
 * default stream).  `max_tensor_elems` bounds one tensor (<= EXCP_MAX_TENSOR_ELEMS);
 * `max_group_elems` (>= max_tensor_elems) is how many elements are processed together: the
 * workspace is about 25 bytes per group element, and a larger batch is run as several groups. */
int excp_create(excp_ctx **out, int hip_device, void *hip_stream,
                uint64_t max_tensor_elems, uint64_t max_group_elems);
void excp_destroy(excp_ctx *ctx);

/* Worst-case compressed size of an n-element tensor (every element kept).  nbits in [2,8], or 32 for
 * EXCP_FLAG_NO_QUANT; 0 for any other nbits. */
uint64_t excp_blob_bound(uint64_t n, int nbits);
/* Exact compressed size for given counts (the closed form of the layout above). */
uint64_t excp_blob_size(uint64_t n, uint64_t n_w, uint64_t n_o, int nbits);
/* The same for a blob written with `flags` (nbits = 32 with EXCP_FLAG_NO_QUANT; the larger second
 * bitmap with EXCP_FLAG_NO_W2M); 0 for inconsistent arguments. */
uint64_t excp_blob_size_ex(uint64_t n, uint64_t n_w, uint64_t n_o, int nbits, uint32_t flags);

/* Alg. 1 (minus the archive step) for `count` tensors; asynchronous.  flags: 0 or EXCP_FLAG_* ORed. */
int excp_compress_tensors(excp_ctx *ctx, int count, const excp_tensor *tensors,
                          float alpha, float beta, int nbits, int lloyd_iters, uint32_t flags);

/* Alg. 2 for `count` tensors; asynchronous. */
int excp_decompress_tensors(excp_ctx *ctx, int count, const excp_blob *blobs);

/* Alg. 3 for `count` tensors; asynchronous.  The weights are read once and written once however
 * long the chain is; every checkpoint adds its centres with one fp32 addition per kept element, so
 * the result equals `steps` applications of Alg. 2 bit for bit.  EXCP_E_ARG if a chain is longer than
 * EXCP_MAX_CHAIN or if all chains together hold more than 4096 checkpoints.
 * After excp_collect a tensor's status is that of its first damaged checkpoint; n_w, n_o and
 * blob_bytes are those of its last one. */
int excp_reconstruct_chain(excp_ctx *ctx, int count, const excp_chain *chains);

/* The stored layout of Sec. 4.2 ("dense"): one code per ELEMENT, 0 = pruned, 1..2^nbits-1 = centre
 * index + 1 -- the tensors Alg. 1 hands to its general-purpose archiver.  Codes of nbits <= 4 sit two
 * to a byte, the even element in the low four bits (the paper does not say which half; an odd
 * tensor leaves the last high half zero); wider codes take one byte each.  The header and the
 * three codebooks travel beside them as the first excp_head_bytes(nbits) bytes of the blob. */
uint64_t excp_dense_bytes(uint64_t n, int nbits);   /* bytes of one code tensor */
uint64_t excp_head_bytes(int nbits);                /* 80 + 12 * 2^nbits; 0 for nbits outside [2,8] */

/* One tensor of an export batch: blob -> per-element code tensors. */
typedef struct {
    const void *blob;            /* device, 16-B aligned */
    uint64_t    blob_bytes;      /* bytes readable at blob */
    uint64_t    n;               /* must equal the n stored in the blob */
    void       *head;            /* device, 16-B aligned, nullable: receives excp_head_bytes(nbits) bytes */
    uint8_t    *codes_w;         /* device, 16-B aligned, nullable: excp_dense_bytes(n, nbits) bytes each; */
    uint8_t    *codes_m;         /*   every byte is written (pruned elements as code 0)                    */
    uint8_t    *codes_v;
} excp_dense_export;

/* One tensor of a reconstruction from that layout (Alg. 2 on per-element codes). */
typedef struct {
    const void    *W_prev_recon; /* device, n weights; needed when W_recon_out is given */
    const void    *head;         /* device, 16-B aligned: header and codebooks */
    uint64_t       head_bytes;   /* bytes readable at head */
    uint64_t       n;            /* must equal the n stored in the header */
    const uint8_t *codes_w;      /* device, 16-B aligned; each needed when its output is given */
    const uint8_t *codes_m;
    const uint8_t *codes_v;
    void          *W_recon_out;  /* device, n weights, nullable; may equal W_prev_recon */
    float         *m_out;        /* device, n, nullable */
    float         *v_out;        /* device, n, nullable */
    uint32_t       flags;        /* storage of the weight arrays, as in excp_blob */
    uint32_t       reserved;     /* 0 */
} excp_dense_blob;

/* Blob -> the layout of Sec. 4.2, for `count` tensors; asynchronous, results by excp_collect (n,
 * n_w, n_o, blob_bytes, status as after a decompress batch; EXCP_E_BLOB for a damaged blob). */
int excp_export_dense(excp_ctx *ctx, int count, const excp_dense_export *items);

/* Alg. 2 from the layout of Sec. 4.2, for `count` tensors; asynchronous.  W_hat[i] = W_prev_recon[i]
 * + C_w[code] where the code is non-zero, else W_prev_recon[i] unchanged; moments C[code] or +0.
 * Bit-identical to excp_decompress_tensors on the blob the codes were exported from.  EXCP_E_BLOB
 * (by excp_collect) for a bad header, a code beyond the codebook or a set unused half-byte; the
 * counts n_w, n_o reported are those stored in the header and are not re-counted. */
int excp_decompress_dense(excp_ctx *ctx, int count, const excp_dense_blob *items);

/* Wait for the pending batch; fill stats[0..count) (nullable); return EXCP_OK or the first
 * per-tensor error.  After a decompress batch only n, n_w, n_o, blob_bytes and status are set. */
int excp_collect(excp_ctx *ctx, excp_stats *stats);

/* Single-tensor forms (Alg. 1 / Alg. 2 argument lists); they wait for completion.
 * blob_bytes and stats are host pointers and may be NULL.  The flags of excp_decompress_step are
 * those of excp_blob (the storage of the weight arrays). */
int excp_compress_step(excp_ctx *ctx,
                       const void *W_prev_recon, const void *W_t, const float *m_t, const float *v_t,
                       uint64_t n, float alpha, float beta, int nbits, int lloyd_iters, uint32_t flags,
                       void *blob_out, uint64_t blob_cap, uint64_t *blob_bytes,
                       void *W_recon_out, excp_stats *stats);
int excp_decompress_step(excp_ctx *ctx, const void *W_prev_recon, const void *blob, uint64_t blob_bytes,
                         uint64_t n, void *W_recon_out, float *m_out, float *v_out, uint32_t flags);

/* For callers that cannot allocate -- code under HIP graph capture restrictions, tight serving loops,
 * harnesses that forbid hipMalloc: Alg. 2 for one tensor exactly as excp_decompress_step computes it,
 * without a context and without allocating anything, on the device or on the host.  The tables the
 * decoding kernels keep between their launches (the tensor's descriptor and state, per-tile survivor
 * counts of both bitmaps, the result record: about 0.5 MiB) live in a static device array inside the
 * library, one copy per GPU, held until the process ends; that fixes the largest tensor:
 * n <= EXCP_STATIC_MAX_ELEMS, EXCP_E_ARG beyond it (larger tensors: a context).  Work is enqueued on
 * `hip_stream` (a hipStream_t, borrowed; NULL = the default stream) of device `hip_device`, and the
 * call waits for it.  Arguments, outputs, flags and errors are those of excp_decompress_step (blobs
 * written with EXCP_FLAG_NO_QUANT are read too).  Every call on one GPU uses that GPU's one array:
 * calls that overlap on the same GPU, from any threads or streams, race -- serialise them.  Calls on
 * different GPUs are independent. */
#define EXCP_STATIC_MAX_ELEMS 268435456ull   /* 2^28 */
int excp_decompress_step_static(int hip_device, void *hip_stream, const void *W_prev_recon, const void *blob,
                                uint64_t blob_bytes, uint64_t n, void *W_recon_out, float *m_out, float *v_out,
                                uint32_t flags);

/* Per-stage timing.  When enabled, HIP events bracket every kernel stage of the next batches;
 * after excp_collect, excp_stage_ms returns the summed milliseconds and launches of stage `i`
 * (0 <= i < excp_stage_count()); excp_stage_name names it. */
int         excp_set_profiling(excp_ctx *ctx, int enabled);
int         excp_stage_count(void);
const char *excp_stage_name(int i);
int         excp_stage_ms(excp_ctx *ctx, int i, double *ms, int *launches);

/* Size thresholds at which the library switches between forms of its kernels.  The forms compute the
 * same bytes; the thresholds only decide which is faster, and the defaults are the measured ones.  They
 * are settable so that the forms meant for very large tensors can be exercised -- and compared with a
 * CPU reference -- on tensors a host can process.  value > 0; not while a batch is pending.
 *   EXCP_PARAM_WIDE_ELEMS      (default 2^28): a group holding a tensor of at least this many elements
 *                              computes the per-bucket totals and initial centres of Sec. 3.3 with
 *                              sixteen waves and one workgroup per bucket.
 *   EXCP_PARAM_CAND_LIST_ELEMS (default 2^26): a tensor's median candidates (Sec. 3.2) are filed in
 *                              n / value lists (at least 1, at most 16), each with a counter of its own. */
#define EXCP_PARAM_WIDE_ELEMS       1
#define EXCP_PARAM_CAND_LIST_ELEMS  2
int excp_set_param(excp_ctx *ctx, int param, uint64_t value);

/* Measurement aid, not part of the method: a plain device-to-device copy of nbytes (multiple of 16,
 * both pointers 16-B aligned) on the context's stream, asynchronous.  Its HBM traffic is exactly nbytes
 * read and nbytes written, which is what bench.py and the profile summaries calibrate a profiler's byte
 * counters with. */
int excp_copy_probe(excp_ctx *ctx, void *dst, const void *src, uint64_t nbytes);

/* Bytes of device workspace the context holds. */
uint64_t excp_workspace_bytes(const excp_ctx *ctx);

const char *excp_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* EXCP_H */
