// Host side of the ExCP library: argument checks, grouping of tensors, workspace, launch order
// (Alg. 1 and Alg. 2), result collection.  No computation of the method happens here.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <algorithm>
#include <mutex>
#include <vector>

#include "../../include/excp.h"
#include "excp_device.h"

namespace {

constexpr u32 kMaxGroupTensors = 1024;   // tensors processed together (== EXCP_MAX_GROUP_TENSORS of the kernels)
constexpr u32 kMaxBatchTensors = 4096;   // tensors per compress / decompress call

enum Stage {
    ST_SAMPLE = 0, ST_STATS, ST_SELECT, ST_SELECT_FALLBACK, ST_MASK_COMPACT, ST_MASK_SCAN, ST_MASK_GATHER, ST_LAYOUT, ST_KM_SAMPLE, ST_KM_COUNT, ST_KM_SCAN,
    ST_KM_SCATTER, ST_KM_BUCKET_STATS, ST_KM_INIT, ST_KM_CLASSIFY, ST_KM_ITER, ST_KM_UPDATE, ST_ASSIGN_PACK, ST_FINALIZE,
    ST_DECODE_PREP, ST_DECODE_MAIN, ST_EXPORT_DENSE, ST_DECODE_DENSE, ST_MISC, ST_COUNT
};
const char *kStageNames[ST_COUNT] = {
    "median_sample", "stats_stream", "select_candidates", "select_fallback", "mask_slots", "mask_scan", "mask_gather", "layout", "km_sample", "km_count", "km_scan",
    "km_scatter", "km_bucket_stats", "km_init", "km_classify", "km_iter", "km_update", "assign_pack", "finalize",
    "decode_prep", "decode_main", "export_dense", "decode_dense", "misc"};

struct Span { int stage; hipEvent_t a, b; };
struct Group { u32 first, count, ntiles; };
struct CGroup { u32 first, count, first_desc, ndescs, ntiles, tb_desc, tb_chain; };

constexpr size_t kEventPool = 8192;      // events made by excp_set_profiling: 4096 timed stages per batch

}  // namespace

struct excp_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    u64 max_tensor = 0, max_group = 0, max_tiles = 0;
    Workspace w{};
    // per-batch arrays (device) and their pinned staging (host)
    TDesc *desc_all = nullptr; TState *st_all = nullptr; u32 *cand_ctr_all = nullptr;
    DDesc *ddesc_all = nullptr; DState *dst_all = nullptr;
    CDesc *cdesc_all = nullptr; CDesc *h_cdesc = nullptr;
    u32 *tile_begin_all = nullptr;
    TDesc *h_desc = nullptr; DDesc *h_ddesc = nullptr; u32 *h_tile_begin = nullptr; HostRec *h_rec = nullptr;
    int *h_err = nullptr;
    u64 status_words = 0;
    u64 ws_bytes = 0;
    std::vector<void *> allocs;
    // pending batch
    int pending = 0;      // 0 none, 1 compress, 2 decompress
    int pending_count = 0;
    bool broken = false;  // a HIP call failed while a batch was being enqueued: the context takes no more work
    // per-call lists; their storage is reserved in excp_create so that no call allocates
    std::vector<Group> groups;
    std::vector<CGroup> cgroups;
    std::vector<u32> tb_offsets;
    // size thresholds of the kernel forms (excp_set_param)
    u64 wide_elems = 1ull << 28;        // a group with a tensor this large takes the sixteen-wave per-bucket kernels
    u64 cand_list_elems = 1ull << 26;   // one median-candidate list per this many elements of a tensor (1 .. 16 lists)
    // profiling
    bool profiling = false;
    std::vector<Span> spans;
    std::vector<hipEvent_t> free_events;
    double stage_ms[ST_COUNT] = {0};
    int stage_launches[ST_COUNT] = {0};
};

namespace {

template <class T>
bool dev_alloc(excp_ctx *c, T **p, u64 count) {
    u64 bytes = count * sizeof(T);
    if (bytes == 0) bytes = 16;
    void *q = nullptr;
    if (hipMalloc(&q, bytes) != hipSuccess) return false;
    c->allocs.push_back(q);
    c->ws_bytes += bytes;
    *p = (T *)q;
    return true;
}

struct StageTimer {
    excp_ctx *c; int stage; hipEvent_t a = nullptr, b = nullptr;
    StageTimer(excp_ctx *ctx, int st) : c(ctx), stage(st) {
        if (!c->profiling) return;
        // events come from the pool excp_set_profiling made; a batch with more stages than the pool
        // holds leaves the rest untimed rather than create events in the middle of a step
        if (c->free_events.size() < 2) return;
        a = c->free_events.back(); c->free_events.pop_back();
        b = c->free_events.back(); c->free_events.pop_back();
        (void)hipEventRecord(a, c->stream);
    }
    ~StageTimer() {
        if (!c->profiling || !a || !b) return;
        (void)hipEventRecord(b, c->stream);
        c->spans.push_back({stage, a, b});
    }
};

// A HIP call failed after part of a batch was enqueued.  The copies already queued read the pinned
// staging arrays, so the stream is drained before anything may overwrite them, and the context takes
// no further work: what state the device tables are in is unknown.
int enqueue_failed(excp_ctx *c) {
    (void)hipStreamSynchronize(c->stream);
    (void)hipGetLastError();
    for (auto &sp : c->spans) { c->free_events.push_back(sp.a); c->free_events.push_back(sp.b); }
    c->spans.clear();
    c->pending = 0;
    c->broken = true;
    return EXCP_E_HIP;
}

u64 blob_size_host(u64 n, u64 nw, u64 no, int nbits, u32 flags = 0) {
    u64 s = EXCP_HEADER + excp_books_bytes((u32)nbits);
    s += excp_pad16(8 * excp_words(n));
    s += excp_pad16(8 * excp_words((flags & EXCP_FLAG_NO_W2M) ? n : nw));
    s += excp_pad16(8 * excp_words(nw * (u64)nbits));
    s += 2 * excp_pad16(8 * excp_words(no * (u64)nbits));
    return s;
}

// Split [0, count) into groups: at most kMaxGroupTensors tensors, cap_elems elements, tcap tensors.
template <class GetN>
void make_groups(int count, u64 cap_elems, u32 tcap, GetN get_n, std::vector<Group> &out) {
    u32 i = 0;
    while (i < (u32)count) {
        Group g{i, 0, 0};
        u64 elems = 0;
        while (i < (u32)count && g.count < tcap) {
            u64 n = get_n(i);
            if (g.count && elems + n > cap_elems) break;
            elems += n;
            g.ntiles += (u32)((n + EXCP_TILE - 1) / EXCP_TILE);
            ++g.count; ++i;
        }
        out.push_back(g);
    }
}

void run_decode_prep_and_main(excp_ctx *c, const Workspace &w, u32 ntensors, u32 ntiles, bool moments) {
    {
        StageTimer t(c, ST_DECODE_PREP);
        launch_decode_count(w, ntensors, ntiles, 0, c->stream);
        launch_decode_scan(w, ntensors, 0, c->stream);
        if (moments) {
            launch_decode_count(w, ntensors, ntiles, 1, c->stream);
            launch_decode_scan(w, ntensors, 1, c->stream);
        }
    }
    {
        StageTimer t(c, ST_DECODE_MAIN);
        launch_decode_main(w, ntensors, ntiles, moments, c->stream);
        launch_decode_main16(w, ntensors, ntiles, moments, c->stream);  // blobs of 16-bit weights, if any
        launch_decode_raw(w, ntensors, ntiles, moments, c->stream);     // blobs written without quantisation, if any
    }
}

// Shared by the two calls that work on the per-element code tensors of Sec. 4.2.  `fill` writes the
// descriptor of tensor i (everything but the tile fields).
template <class Fill>
int run_dense(excp_ctx *c, int count, bool exporting, Fill fill) {
    if (hipSetDevice(c->device) != hipSuccess) return EXCP_E_HIP;
    std::vector<Group> &groups = c->groups;
    std::vector<u32> &tb_offsets = c->tb_offsets;
    groups.clear(); tb_offsets.clear();
    make_groups(count, c->max_group, kMaxGroupTensors, [&](u32 i) { DDesc d; fill(i, d); return (u64)d.n; }, groups);
    u32 tb_off = 0;
    for (const Group &g : groups) {
        u32 tile = 0;
        tb_offsets.push_back(tb_off);
        for (u32 q = 0; q < g.count; ++q) {
            DDesc &d = c->h_ddesc[g.first + q];
            fill(g.first + q, d);
            d.tile_begin = tile; d.tile_count = (u32)((d.n + EXCP_TILE - 1) / EXCP_TILE);
            c->h_tile_begin[tb_off + q] = tile;
            tile += d.tile_count;
        }
        c->h_tile_begin[tb_off + g.count] = tile;
        tb_off += g.count + 1;
    }
    hipStream_t s = c->stream;
    if (count) {
        if (hipMemcpyAsync(c->ddesc_all, c->h_ddesc, sizeof(DDesc) * count, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(c->tile_begin_all, c->h_tile_begin, sizeof(u32) * tb_off, hipMemcpyHostToDevice, s) != hipSuccess)
            return enqueue_failed(c);
    }
    for (size_t gi = 0; gi < groups.size(); ++gi) {
        const Group &g = groups[gi];
        Workspace w = c->w;
        w.ddesc = c->ddesc_all + g.first;
        w.dst = c->dst_all + g.first;
        w.tile_begin = c->tile_begin_all + tb_offsets[gi];
        w.rec_dev = c->w.rec_dev + g.first;
        w.rec_base = 0;
        if (exporting) {
            { StageTimer t(c, ST_MISC); launch_decode_parse(w, g.count, false, s); }
            bool moments = false;
            for (u32 q = 0; q < g.count; ++q)
                moments = moments || c->h_ddesc[g.first + q].cm != nullptr || c->h_ddesc[g.first + q].cv != nullptr;
            {
                StageTimer t(c, ST_DECODE_PREP);
                launch_decode_count(w, g.count, g.ntiles, 0, s);
                launch_decode_scan(w, g.count, 0, s);
                if (moments) {
                    launch_decode_count(w, g.count, g.ntiles, 1, s);
                    launch_decode_scan(w, g.count, 1, s);
                }
            }
            { StageTimer t(c, ST_EXPORT_DENSE); launch_export_dense(w, g.count, g.ntiles, moments, s); }
        } else {
            { StageTimer t(c, ST_MISC); launch_dense_parse(w, g.count, s); }
            { StageTimer t(c, ST_DECODE_DENSE); launch_decode_dense(w, g.count, g.ntiles, s); }
        }
        { StageTimer t(c, ST_MISC); launch_decode_finish(w, g.count, s); }
    }
    if (count) {
        if (hipMemcpyAsync(c->h_rec, c->w.rec_dev, sizeof(HostRec) * count, hipMemcpyDeviceToHost, s) != hipSuccess)
            return enqueue_failed(c);
    }
    if (hipMemcpyAsync(c->h_err, c->w.err_flag, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess) return enqueue_failed(c);
    if (hipGetLastError() != hipSuccess) return enqueue_failed(c);
    c->pending = 2;
    c->pending_count = count;
    return EXCP_OK;
}

// ---- Alg. 2 for one tensor without any allocation -------------------------------------------------
// Everything the decoders keep between their kernels -- the descriptor and state of the tensor, its
// two-entry tile table, the per-tile survivor counts of both bitmaps, the scan's part totals, the
// result record -- lives in one file-scope device array instead of a context's workspace.  Every GPU
// has its own copy of the array at its own address: the address is asked for once per device and kept.
constexpr u64 kStaticMaxTiles = EXCP_STATIC_MAX_ELEMS / EXCP_TILE;
struct StaticOffsets {
    static constexpr u64 ddesc = 0, dst = 256, tile_begin = 512, dec_kinds = 768, rec = 1024, dec_part = 1280,
                         cnt_w = 1536, cnt_o = cnt_w + 4 * (kStaticMaxTiles + 64), end = cnt_o + 4 * (kStaticMaxTiles + 64);
};
static_assert(sizeof(DDesc) <= 256 && sizeof(DState) <= 256 && sizeof(HostRec) <= 256, "scratch slots are 256 bytes");
static_assert(StaticOffsets::cnt_w % 256 == 0 && StaticOffsets::cnt_o % 256 == 0, "tables start on 256-byte boundaries");
constexpr u64 kScratchBytes = StaticOffsets::end;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
struct StaticDevice { unsigned char *ptr = nullptr; int cus = 0; bool ready = false; };
StaticDevice g_static[kMaxDevices];
std::mutex g_static_mutex;

// The device's copy of `scratch` and its compute-unit count, looked up on the first call per device
// (with that device current).  The array's name is only a handle on the host; kernels and copies are
// given the address returned here.
int static_device(int device, StaticDevice &out) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticDevice &d = g_static[device];
    if (!d.ready) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return EXCP_E_HIP;
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, device) != hipSuccess || prop.multiProcessorCount <= 0) return EXCP_E_HIP;
        d.ptr = (unsigned char *)p; d.cus = prop.multiProcessorCount; d.ready = true;
    }
    out = d;
    return EXCP_OK;
}

}  // namespace

extern "C" {

const char *excp_strerror(int code) {
    switch (code) {
        case EXCP_OK: return "ok";
        case EXCP_E_ARG: return "invalid argument";
        case EXCP_E_CAP: return "blob capacity too small";
        case EXCP_E_NONFINITE: return "non-finite input";
        case EXCP_E_BLOB: return "malformed compressed tensor";
        case EXCP_E_HIP: return "HIP error";
        case EXCP_E_STATE: return "call order violated";
        case EXCP_E_INTERNAL: return "internal work list overflowed";
        default: return "unknown error";
    }
}

uint64_t excp_blob_size(uint64_t n, uint64_t n_w, uint64_t n_o, int nbits) {
    if (((nbits < 2 || nbits > 8) && nbits != (int)EXCP_RAW_BITS) || n_w > n || n_o > n_w) return 0;
    return blob_size_host(n, n_w, n_o, nbits);
}

uint64_t excp_blob_size_ex(uint64_t n, uint64_t n_w, uint64_t n_o, int nbits, uint32_t flags) {
    const bool raw = (flags & EXCP_FLAG_NO_QUANT) != 0, nw2m = (flags & EXCP_FLAG_NO_W2M) != 0;
    if (flags > 63u || (flags & 0x30u) == 0x30u || (raw ? nbits != (int)EXCP_RAW_BITS : (nbits < 2 || nbits > 8))) return 0;
    if (n_w > n || n_o > (nw2m ? n : n_w)) return 0;
    return blob_size_host(n, n_w, n_o, nbits, flags);
}

uint64_t excp_blob_bound(uint64_t n, int nbits) {
    if ((nbits < 2 || nbits > 8) && nbits != (int)EXCP_RAW_BITS) return 0;
    return blob_size_host(n, n, n, nbits);
}

int excp_stage_count(void) { return ST_COUNT; }
const char *excp_stage_name(int i) { return (i >= 0 && i < ST_COUNT) ? kStageNames[i] : ""; }

int excp_create(excp_ctx **out, int hip_device, void *hip_stream, uint64_t max_tensor_elems,
                uint64_t max_group_elems) {
    if (!out) return EXCP_E_ARG;
    *out = nullptr;
    if (max_tensor_elems == 0 || max_tensor_elems > EXCP_MAX_TENSOR_ELEMS) return EXCP_E_ARG;
    if (max_group_elems < max_tensor_elems) return EXCP_E_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || hip_device < 0 || hip_device >= ndev) return EXCP_E_HIP;
    if (hipSetDevice(hip_device) != hipSuccess) return EXCP_E_HIP;
    excp_ctx *c = new (std::nothrow) excp_ctx();
    if (!c) return EXCP_E_HIP;
    c->device = hip_device;
    c->stream = (hipStream_t)hip_stream;
    c->max_tensor = max_tensor_elems;
    c->max_group = max_group_elems;
    try {                                     // every list a later call fills is reserved here, at its largest
        c->groups.reserve(kMaxBatchTensors);
        c->cgroups.reserve(kMaxBatchTensors);
        c->tb_offsets.reserve(kMaxBatchTensors);
        c->spans.reserve(kEventPool / 2);
        c->free_events.reserve(kEventPool);
    } catch (...) { delete c; return EXCP_E_HIP; }
    Workspace &w = c->w;
    const u64 G = max_group_elems;
    const u64 max_tiles = G / EXCP_TILE + kMaxGroupTensors + 1;
    const u64 chunks_group = 3 * (G / EXCP_CHUNK) + 3 * kMaxGroupTensors + 3;
    c->status_words = max_tiles;
    c->max_tiles = max_tiles;
    bool ok = true;
    ok = ok && dev_alloc(c, &c->desc_all, kMaxBatchTensors);
    ok = ok && dev_alloc(c, &c->st_all, kMaxBatchTensors);
    ok = ok && dev_alloc(c, &c->cand_ctr_all, (u64)kMaxBatchTensors * 512);
    ok = ok && dev_alloc(c, &c->ddesc_all, kMaxBatchTensors);
    ok = ok && dev_alloc(c, &c->dst_all, kMaxBatchTensors);
    ok = ok && dev_alloc(c, &c->cdesc_all, kMaxBatchTensors);
    ok = ok && dev_alloc(c, &c->tile_begin_all, (u64)kMaxBatchTensors * 2 + 16);
    ok = ok && dev_alloc(c, &w.seg, 3ull * kMaxGroupTensors);
    ok = ok && dev_alloc(c, &w.xw, G);
    ok = ok && dev_alloc(c, &w.xm, G);
    ok = ok && dev_alloc(c, &w.xv, G);
    ok = ok && dev_alloc(c, &w.med_hist, (u64)kMaxGroupTensors * 2048);
    ok = ok && dev_alloc(c, &w.cand, G / 12 + 4096ull * kMaxGroupTensors + 16);
    ok = ok && dev_alloc(c, &w.tile_status, 2 * max_tiles);      // one word per 2048-element sub-tile
    ok = ok && dev_alloc(c, &w.mask_prefix, 2 * max_tiles);
    ok = ok && dev_alloc(c, &w.mask_part, (u64)kMaxGroupTensors * 16);
    ok = ok && dev_alloc(c, &w.mask_bo, 2 * max_tiles * 32);
    ok = ok && dev_alloc(c, &w.chunk_total, 4);
    ok = ok && dev_alloc(c, &w.seg_chunk_begin, 3ull * kMaxGroupTensors + 4);
    const u64 nseg_max = 3ull * kMaxGroupTensors;
    const u64 acc_words = nseg_max * EXCP_MAX_K * (EXCP_ABSM_BINS + 1);
    ok = ok && dev_alloc(c, &w.pw, G);
    ok = ok && dev_alloc(c, &w.pm, G);
    ok = ok && dev_alloc(c, &w.pv, G);
    ok = ok && dev_alloc(c, &w.km_split, nseg_max * EXCP_KM_MAP_WORDS);
    ok = ok && dev_alloc(c, &w.km_cnt, chunks_group * 256);
    ok = ok && dev_alloc(c, &w.km_begin, nseg_max * 257);
    ok = ok && dev_alloc(c, &w.km_part, nseg_max * 16 * 256);
    ok = ok && dev_alloc(c, &w.km_bsum, nseg_max * 256 * EXCP_ABSM_BINS);
    ok = ok && dev_alloc(c, &w.km_min, nseg_max * 256);
    ok = ok && dev_alloc(c, &w.km_max, nseg_max * 256);
    ok = ok && dev_alloc(c, &w.km_acc, acc_words);
    const u64 item_cap = chunks_group + nseg_max * 256;
    ok = ok && dev_alloc(c, (unsigned char **)&w.km_items, item_cap * 16);
    ok = ok && dev_alloc(c, &w.km_item_count, 4);
    w.km_item_cap = (u32)(item_cap > 0xffffffffull ? 0xffffffffull : item_cap);
    ok = ok && dev_alloc(c, &w.part_obj, chunks_group);
    // per-tile survivor counts of decode; a chain reconstruction keeps those of all its checkpoints
    ok = ok && dev_alloc(c, &w.dec_cnt_w, max_tiles * EXCP_MAX_CHAIN);
    ok = ok && dev_alloc(c, &w.dec_cnt_o, max_tiles * EXCP_MAX_CHAIN);
    ok = ok && dev_alloc(c, &w.dec_kinds, 4);
    ok = ok && dev_alloc(c, &w.dec_part, (u64)kMaxGroupTensors * 16);
    ok = ok && dev_alloc(c, &w.err_flag, 4);
    ok = ok && dev_alloc(c, &w.rec_dev, kMaxBatchTensors);
    w.max_chunks = (u32)(chunks_group > 0xffffffffull ? 0xffffffffull : chunks_group);
    if (ok) {
        ok = hipHostMalloc((void **)&c->h_desc, sizeof(TDesc) * kMaxBatchTensors) == hipSuccess &&
             hipHostMalloc((void **)&c->h_ddesc, sizeof(DDesc) * kMaxBatchTensors) == hipSuccess &&
             hipHostMalloc((void **)&c->h_cdesc, sizeof(CDesc) * kMaxBatchTensors) == hipSuccess &&
             hipHostMalloc((void **)&c->h_tile_begin, sizeof(u32) * (kMaxBatchTensors * 2 + 16)) == hipSuccess &&
             hipHostMalloc((void **)&c->h_rec, sizeof(HostRec) * kMaxBatchTensors) == hipSuccess &&
             hipHostMalloc((void **)&c->h_err, 16) == hipSuccess;
    }
    if (ok) {
        hipDeviceProp_t prop;
        ok = hipGetDeviceProperties(&prop, hip_device) == hipSuccess && prop.multiProcessorCount > 0;
        w.cus = ok ? prop.multiProcessorCount : 0;
    }
    if (ok) {
        launch_zero_u32(w.med_hist, (u64)kMaxGroupTensors * 2048, c->stream);
        launch_zero_u32((u32 *)w.km_acc, 2 * acc_words, c->stream);
        launch_zero_u32(w.km_item_count, 4, c->stream);
        launch_zero_u32((u32 *)w.err_flag, 4, c->stream);
        ok = hipStreamSynchronize(c->stream) == hipSuccess;
    }
    if (!ok) { excp_destroy(c); return EXCP_E_HIP; }
    *out = c;
    return EXCP_OK;
}

void excp_destroy(excp_ctx *c) {
    if (!c) return;
    (void)hipSetDevice(c->device);
    (void)hipStreamSynchronize(c->stream);
    for (void *p : c->allocs) (void)hipFree(p);
    if (c->h_desc) (void)hipHostFree(c->h_desc);
    if (c->h_ddesc) (void)hipHostFree(c->h_ddesc);
    if (c->h_cdesc) (void)hipHostFree(c->h_cdesc);
    if (c->h_tile_begin) (void)hipHostFree(c->h_tile_begin);
    if (c->h_rec) (void)hipHostFree(c->h_rec);
    if (c->h_err) (void)hipHostFree(c->h_err);
    for (auto &s : c->spans) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
    for (auto e : c->free_events) (void)hipEventDestroy(e);
    delete c;
}

uint64_t excp_workspace_bytes(const excp_ctx *c) { return c ? c->ws_bytes : 0; }

int excp_copy_probe(excp_ctx *c, void *dst, const void *src, uint64_t nbytes) {
    if (!c || !dst || !src || (nbytes & 15u) || (((uintptr_t)dst | (uintptr_t)src) & 15u)) return EXCP_E_ARG;
    if (hipSetDevice(c->device) != hipSuccess) return EXCP_E_HIP;
    launch_copy_probe(src, dst, nbytes, c->stream);
    return hipGetLastError() == hipSuccess ? EXCP_OK : EXCP_E_HIP;
}

int excp_set_profiling(excp_ctx *c, int enabled) {
    if (!c) return EXCP_E_ARG;
    if (c->pending) return EXCP_E_STATE;
    if (c->broken) return EXCP_E_HIP;
    if (enabled && c->free_events.empty()) {
        // the event pool is made here, once, so that no timed step creates events
        if (hipSetDevice(c->device) != hipSuccess) return EXCP_E_HIP;
        for (size_t i = 0; i < kEventPool; ++i) {
            hipEvent_t e = nullptr;
            if (hipEventCreate(&e) != hipSuccess) return EXCP_E_HIP;
            c->free_events.push_back(e);
        }
    }
    c->profiling = enabled != 0;
    return EXCP_OK;
}

int excp_set_param(excp_ctx *c, int param, uint64_t value) {
    if (!c || value == 0) return EXCP_E_ARG;
    if (c->pending) return EXCP_E_STATE;
    switch (param) {
        case EXCP_PARAM_WIDE_ELEMS: c->wide_elems = value; return EXCP_OK;
        case EXCP_PARAM_CAND_LIST_ELEMS: c->cand_list_elems = value; return EXCP_OK;
        default: return EXCP_E_ARG;
    }
}

int excp_stage_ms(excp_ctx *c, int i, double *ms, int *launches) {
    if (!c || i < 0 || i >= ST_COUNT) return EXCP_E_ARG;
    if (ms) *ms = c->stage_ms[i];
    if (launches) *launches = c->stage_launches[i];
    return EXCP_OK;
}

int excp_compress_tensors(excp_ctx *c, int count, const excp_tensor *tensors, float alpha, float beta,
                          int nbits, int lloyd_iters, uint32_t flags) {
    if (!c || count < 0 || (count && !tensors)) return EXCP_E_ARG;
    if (c->pending) return EXCP_E_STATE;
    if (c->broken) return EXCP_E_HIP;
    if ((u32)count > kMaxBatchTensors) return EXCP_E_ARG;
    if (nbits < 2 || nbits > 8 || lloyd_iters < 0 || (flags & ~63u) != 0 || (flags & 0x30u) == 0x30u) return EXCP_E_ARG;
    if (!(alpha >= 0.f) || !(beta >= 0.f) || isinf(alpha) || isinf(beta)) return EXCP_E_ARG;
    const bool raw = (flags & EXCP_FLAG_NO_QUANT) != 0;     // survivors stored as fp32: no codebook stage at all
    if (raw) nbits = (int)EXCP_RAW_BITS;
    const int K = raw ? 0 : (1 << nbits) - 1;
    for (int i = 0; i < count; ++i) {
        const excp_tensor &t = tensors[i];
        if (t.n > c->max_tensor) return EXCP_E_ARG;
        if (!t.blob || ((uintptr_t)t.blob & 15u)) return EXCP_E_ARG;
        if (t.n && (!t.W_prev_recon || !t.W_t || !t.m_t || !t.v_t)) return EXCP_E_ARG;
        // the part of the blob whose place does not depend on the data must fit
        if (t.blob_cap < EXCP_HEADER + excp_books_bytes((u32)nbits) + excp_pad16(8 * excp_words(t.n))) return EXCP_E_CAP;
    }
    if (hipSetDevice(c->device) != hipSuccess) return EXCP_E_HIP;
    const u64 cap_elems = c->max_group;
    const u32 tcap = kMaxGroupTensors;
    std::vector<Group> &groups = c->groups;
    std::vector<u32> &tb_offsets = c->tb_offsets;
    groups.clear(); tb_offsets.clear();
    make_groups(count, cap_elems, tcap, [&](u32 i) { return (u64)tensors[i].n; }, groups);

    u32 tb_off = 0;
    for (const Group &g : groups) {
        u64 elem_off = 0, cand_off = 0; u32 tile = 0;
        tb_offsets.push_back(tb_off);
        for (u32 q = 0; q < g.count; ++q) {
            const excp_tensor &t = tensors[g.first + q];
            TDesc &d = c->h_desc[g.first + q];
            d.Wp = (const float *)t.W_prev_recon; d.W = (const float *)t.W_t; d.m = t.m_t; d.v = t.v_t; d.n = t.n;
            d.blob = (unsigned char *)t.blob; d.blob_cap = t.blob_cap; d.W_out = (float *)t.W_recon_out;
            d.elem_off = elem_off; d.tile_begin = tile;
            d.cand_lists = (u32)std::min<u64>(std::max<u64>(t.n / c->cand_list_elems, 1), 16); d.pad0 = 0;
            d.cand_off = cand_off; d.cand_cap = (t.n / 12 + 4096 + d.cand_lists - 1) / d.cand_lists * d.cand_lists;
            cand_off += d.cand_cap;
            d.tile_count = (u32)((t.n + EXCP_TILE - 1) / EXCP_TILE);
            c->h_tile_begin[tb_off + q] = tile;
            elem_off += t.n; tile += d.tile_count;
        }
        c->h_tile_begin[tb_off + g.count] = tile;
        tb_off += g.count + 1;
    }
    hipStream_t s = c->stream;
    if (count) {
        if (hipMemcpyAsync(c->desc_all, c->h_desc, sizeof(TDesc) * count, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(c->tile_begin_all, c->h_tile_begin, sizeof(u32) * tb_off, hipMemcpyHostToDevice, s) != hipSuccess)
            return enqueue_failed(c);
        launch_zero_u32((u32 *)c->st_all, (u64)count * sizeof(TState) / 4, s);
        launch_zero_u32(c->cand_ctr_all, (u64)count * 512, s);
    }
    for (size_t gi = 0; gi < groups.size(); ++gi) {
        const Group &g = groups[gi];
        Workspace w = c->w;
        w.desc = c->desc_all + g.first;
        w.st = c->st_all + g.first;
        w.cand_ctr = c->cand_ctr_all + (u64)g.first * 512;
        w.ddesc = c->ddesc_all + g.first;
        w.dst = c->dst_all + g.first;
        w.tile_begin = c->tile_begin_all + tb_offsets[gi];
        w.rec_base = 0;
        w.rec_dev = c->w.rec_dev + g.first;
        GroupParams p{};
        p.alpha = alpha; p.beta = beta; p.nbits = nbits; p.K = K; p.iters = lloyd_iters; p.flags = flags;
        p.ntensors = g.count; p.ntiles = g.ntiles;
        u64 largest = 0;
        for (u32 q = 0; q < g.count; ++q) largest = std::max<u64>(largest, tensors[g.first + q].n);
        p.wide = largest >= c->wide_elems ? 2u : ((flags & 0x30u) != 0 ? 1u : 0u);
        { StageTimer t(c, ST_SAMPLE); launch_stats(w, p, 0, s); }
        { StageTimer t(c, ST_STATS); launch_stats(w, p, 1, s); }
        {
            StageTimer t(c, ST_SELECT);
            launch_stats(w, p, 2, s);
            for (int pass = 0; pass < 3; ++pass) { launch_stats(w, p, 3, s); launch_stats(w, p, 4, s); }
        }
        {
            StageTimer t(c, ST_SELECT_FALLBACK);     // does nothing unless a sample bracket missed its median
            for (int pass = 0; pass < 3; ++pass) { launch_stats(w, p, 5 + pass, s); launch_stats(w, p, 8 + pass, s); }
            launch_stats(w, p, 11, s);
        }
        { StageTimer t(c, ST_MASK_COMPACT); launch_mask_compact(w, p, 0, s); }
        { StageTimer t(c, ST_MASK_SCAN); launch_mask_compact(w, p, 1, s); }
        { StageTimer t(c, ST_LAYOUT); launch_layout(w, p, s); }
        if (!raw) {
            // the value -> bucket maps come from the slots, and the count table is cleared, before the pass
            // that makes the dense survivor arrays: that pass also takes the bucket counts
            { StageTimer t(c, ST_KM_SAMPLE); launch_km_partition(w, p, 0, s); }
            { StageTimer t(c, ST_KM_COUNT); launch_km_partition(w, p, 1, s); }
        }
        { StageTimer t(c, ST_MASK_GATHER); launch_mask_compact(w, p, 2, s); }
        if (raw) {
            StageTimer t(c, ST_ASSIGN_PACK); launch_store_raw(w, p, s);
        } else {
            { StageTimer t(c, ST_KM_SCAN); launch_km_partition(w, p, 2, s); }
            { StageTimer t(c, ST_KM_SCATTER); launch_km_partition(w, p, 3, s); }
            { StageTimer t(c, ST_KM_BUCKET_STATS); launch_km_partition(w, p, 4, s); }
            { StageTimer t(c, ST_KM_INIT); launch_km_init(w, p, s); }
            for (int it = 0; it < lloyd_iters; ++it) {
                // classification also moves the centres by the previous iteration's totals
                { StageTimer t(c, ST_KM_CLASSIFY); launch_km_classify(w, p, it, s); }
                { StageTimer t(c, ST_KM_ITER); launch_km_iter(w, p, it, s); }
            }
            if (lloyd_iters > 0) { StageTimer t(c, ST_KM_UPDATE); launch_km_update(w, p, s); }
            { StageTimer t(c, ST_ASSIGN_PACK); launch_assign_pack(w, p, s); }
        }
        { StageTimer t(c, ST_FINALIZE); launch_finalize(w, p, s); }
        bool any_out = false;
        for (u32 q = 0; q < g.count; ++q) any_out = any_out || tensors[g.first + q].W_recon_out != nullptr;
        if (any_out) {
            // (the per-tile survivor counts come from the mask pass: no bitmap counting here)
            { StageTimer t(c, ST_MISC); launch_decode_from_compress(w, p, s); }
            StageTimer t(c, ST_DECODE_MAIN);
            if (raw) launch_decode_raw(w, g.count, g.ntiles, false, s);
            else if (flags & 0x30u) launch_decode_main16(w, g.count, g.ntiles, false, s);
            else launch_decode_main(w, g.count, g.ntiles, false, s);
        }
    }
    if (count) {
        if (hipMemcpyAsync(c->h_rec, c->w.rec_dev, sizeof(HostRec) * count, hipMemcpyDeviceToHost, s) != hipSuccess)
            return enqueue_failed(c);
    }
    if (hipMemcpyAsync(c->h_err, c->w.err_flag, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess) return enqueue_failed(c);
    if (hipGetLastError() != hipSuccess) return enqueue_failed(c);
    c->pending = 1;
    c->pending_count = count;
    return EXCP_OK;
}

int excp_decompress_tensors(excp_ctx *c, int count, const excp_blob *blobs) {
    if (!c || count < 0 || (count && !blobs)) return EXCP_E_ARG;
    if (c->pending) return EXCP_E_STATE;
    if (c->broken) return EXCP_E_HIP;
    if ((u32)count > kMaxBatchTensors) return EXCP_E_ARG;
    for (int i = 0; i < count; ++i) {
        const excp_blob &b = blobs[i];
        if ((b.flags & ~0x30u) || (b.flags & 0x30u) == 0x30u) return EXCP_E_ARG;
        if (b.n > c->max_tensor) return EXCP_E_ARG;
        if (!b.blob || ((uintptr_t)b.blob & 15u)) return EXCP_E_ARG;
        if (b.n && !b.W_prev_recon) return EXCP_E_ARG;
    }
    if (hipSetDevice(c->device) != hipSuccess) return EXCP_E_HIP;
    std::vector<Group> &groups = c->groups;
    std::vector<u32> &tb_offsets = c->tb_offsets;
    groups.clear(); tb_offsets.clear();
    make_groups(count, c->max_group, kMaxGroupTensors, [&](u32 i) { return (u64)blobs[i].n; }, groups);
    u32 tb_off = 0;
    for (const Group &g : groups) {
        u32 tile = 0;
        tb_offsets.push_back(tb_off);
        for (u32 q = 0; q < g.count; ++q) {
            const excp_blob &b = blobs[g.first + q];
            DDesc &d = c->h_ddesc[g.first + q];
            d.Wp = (const float *)b.W_prev_recon; d.blob = (const unsigned char *)b.blob; d.blob_bytes = b.blob_bytes; d.n = b.n;
            d.W_out = (float *)b.W_recon_out; d.m_out = b.m_out; d.v_out = b.v_out;
            d.cw = d.cm = d.cv = d.head = nullptr; d.wtype = (b.flags >> 4) & 3u; d.pad = 0;
            d.tile_begin = tile; d.tile_count = (u32)((b.n + EXCP_TILE - 1) / EXCP_TILE);
            c->h_tile_begin[tb_off + q] = tile;
            tile += d.tile_count;
        }
        c->h_tile_begin[tb_off + g.count] = tile;
        tb_off += g.count + 1;
    }
    hipStream_t s = c->stream;
    if (count) {
        if (hipMemcpyAsync(c->ddesc_all, c->h_ddesc, sizeof(DDesc) * count, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(c->tile_begin_all, c->h_tile_begin, sizeof(u32) * tb_off, hipMemcpyHostToDevice, s) != hipSuccess)
            return enqueue_failed(c);
    }
    for (size_t gi = 0; gi < groups.size(); ++gi) {
        const Group &g = groups[gi];
        Workspace w = c->w;
        w.ddesc = c->ddesc_all + g.first;
        w.dst = c->dst_all + g.first;
        w.tile_begin = c->tile_begin_all + tb_offsets[gi];
        w.rec_dev = c->w.rec_dev + g.first;
        w.rec_base = 0;
        { StageTimer t(c, ST_MISC); launch_decode_parse(w, g.count, true, s); }
        bool moments = false;
        for (u32 q = 0; q < g.count; ++q)
            moments = moments || blobs[g.first + q].m_out != nullptr || blobs[g.first + q].v_out != nullptr;
        run_decode_prep_and_main(c, w, g.count, g.ntiles, moments);
        { StageTimer t(c, ST_MISC); launch_decode_finish(w, g.count, s); }
    }
    if (count) {
        if (hipMemcpyAsync(c->h_rec, c->w.rec_dev, sizeof(HostRec) * count, hipMemcpyDeviceToHost, s) != hipSuccess)
            return enqueue_failed(c);
    }
    if (hipMemcpyAsync(c->h_err, c->w.err_flag, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess) return enqueue_failed(c);
    if (hipGetLastError() != hipSuccess) return enqueue_failed(c);
    c->pending = 2;
    c->pending_count = count;
    return EXCP_OK;
}

uint64_t excp_dense_bytes(uint64_t n, int nbits) { return nbits <= 4 ? (n + 1) / 2 : n; }
uint64_t excp_head_bytes(int nbits) { return (nbits < 2 || nbits > 8) ? 0 : EXCP_HEADER + 12ull * (1ull << nbits); }

int excp_export_dense(excp_ctx *c, int count, const excp_dense_export *items) {
    if (!c || count < 0 || (count && !items)) return EXCP_E_ARG;
    if (c->pending) return EXCP_E_STATE;
    if (c->broken) return EXCP_E_HIP;
    if ((u32)count > kMaxBatchTensors) return EXCP_E_ARG;
    for (int i = 0; i < count; ++i) {
        const excp_dense_export &e = items[i];
        if (e.n > c->max_tensor) return EXCP_E_ARG;
        if (!e.blob || ((uintptr_t)e.blob & 15u)) return EXCP_E_ARG;
        if (((uintptr_t)e.head | (uintptr_t)e.codes_w | (uintptr_t)e.codes_m | (uintptr_t)e.codes_v) & 15u) return EXCP_E_ARG;
    }
    return run_dense(c, count, true, [&](u32 i, DDesc &d) {
        const excp_dense_export &e = items[i];
        d.Wp = nullptr; d.blob = (const unsigned char *)e.blob; d.blob_bytes = e.blob_bytes; d.n = e.n;
        d.W_out = d.m_out = d.v_out = nullptr;
        d.cw = e.codes_w; d.cm = e.codes_m; d.cv = e.codes_v; d.head = (unsigned char *)e.head;
        d.wtype = 3u; d.pad = 0;
    });
}

int excp_decompress_dense(excp_ctx *c, int count, const excp_dense_blob *items) {
    if (!c || count < 0 || (count && !items)) return EXCP_E_ARG;
    if (c->pending) return EXCP_E_STATE;
    if (c->broken) return EXCP_E_HIP;
    if ((u32)count > kMaxBatchTensors) return EXCP_E_ARG;
    for (int i = 0; i < count; ++i) {
        const excp_dense_blob &e = items[i];
        if ((e.flags & ~0x30u) || (e.flags & 0x30u) == 0x30u) return EXCP_E_ARG;
        if (e.n > c->max_tensor) return EXCP_E_ARG;
        if (!e.head || ((uintptr_t)e.head & 15u)) return EXCP_E_ARG;
        if (((uintptr_t)e.codes_w | (uintptr_t)e.codes_m | (uintptr_t)e.codes_v) & 15u) return EXCP_E_ARG;
        if (e.n && e.W_recon_out && (!e.W_prev_recon || !e.codes_w)) return EXCP_E_ARG;
        if (e.n && ((e.m_out && !e.codes_m) || (e.v_out && !e.codes_v))) return EXCP_E_ARG;
    }
    return run_dense(c, count, false, [&](u32 i, DDesc &d) {
        const excp_dense_blob &e = items[i];
        d.Wp = (const float *)e.W_prev_recon; d.blob = (const unsigned char *)e.head; d.blob_bytes = e.head_bytes; d.n = e.n;
        d.W_out = (float *)e.W_recon_out; d.m_out = e.m_out; d.v_out = e.v_out;
        d.cw = (unsigned char *)e.codes_w; d.cm = (unsigned char *)e.codes_m; d.cv = (unsigned char *)e.codes_v; d.head = nullptr;
        d.wtype = (e.flags >> 4) & 3u; d.pad = 0;
    });
}

int excp_reconstruct_chain(excp_ctx *c, int count, const excp_chain *chains) {
    if (!c || count < 0 || (count && !chains)) return EXCP_E_ARG;
    if (c->pending) return EXCP_E_STATE;
    if (c->broken) return EXCP_E_HIP;
    if ((u32)count > kMaxBatchTensors) return EXCP_E_ARG;
    u64 total_descs = 0;
    for (int i = 0; i < count; ++i) {
        const excp_chain &ch = chains[i];
        if ((ch.flags & ~0x30u) || (ch.flags & 0x30u) == 0x30u) return EXCP_E_ARG;
        if (ch.n > c->max_tensor || ch.steps < 1 || ch.steps > EXCP_MAX_CHAIN) return EXCP_E_ARG;
        if (!ch.blobs || !ch.blob_bytes) return EXCP_E_ARG;
        if (ch.n && !ch.W0) return EXCP_E_ARG;
        for (int j = 0; j < ch.steps; ++j)
            if (!ch.blobs[j] || ((uintptr_t)ch.blobs[j] & 15u)) return EXCP_E_ARG;
        total_descs += (u64)ch.steps;
    }
    if (total_descs > kMaxBatchTensors) return EXCP_E_ARG;
    if (hipSetDevice(c->device) != hipSuccess) return EXCP_E_HIP;

    // Groups: at most kMaxGroupTensors descriptors (one per tensor and checkpoint) and as many
    // descriptor tiles as the per-tile count tables hold (EXCP_MAX_CHAIN times a group's tiles, so
    // any tensor the context accepts fits with its whole chain).
    std::vector<CGroup> &groups = c->cgroups;
    groups.clear();
    u32 tb_off = 0, desc_off = 0;
    for (u32 i = 0; i < (u32)count;) {
        CGroup g{i, 0, desc_off, 0, 0, 0, 0};
        u64 dtiles = 0;
        while (i < (u32)count) {
            const excp_chain &ch = chains[i];
            const u64 tiles = (ch.n + EXCP_TILE - 1) / EXCP_TILE;
            if (g.count && (g.ndescs + (u32)ch.steps > kMaxGroupTensors || dtiles + tiles * ch.steps > c->max_tiles * EXCP_MAX_CHAIN)) break;
            dtiles += tiles * ch.steps; g.ndescs += (u32)ch.steps; g.ntiles += (u32)tiles; ++g.count; ++i;
        }
        if (tb_off + g.ndescs + g.count + 2 > kMaxBatchTensors * 2 + 16) return EXCP_E_ARG;
        g.tb_desc = tb_off; g.tb_chain = tb_off + g.ndescs + 1;
        u32 dtile = 0, ctile = 0, d = 0;
        for (u32 q = 0; q < g.count; ++q) {
            const excp_chain &ch = chains[g.first + q];
            const u32 tiles = (u32)((ch.n + EXCP_TILE - 1) / EXCP_TILE);
            CDesc &cd = c->h_cdesc[g.first + q];
            cd.W0 = (const float *)ch.W0; cd.W_out = (float *)ch.W_out; cd.n = ch.n; cd.first_desc = d; cd.steps = (u32)ch.steps;
            cd.tile_begin = ctile; cd.tile_count = tiles;
            c->h_tile_begin[g.tb_chain + q] = ctile;
            ctile += tiles;
            for (int j = 0; j < ch.steps; ++j, ++d) {
                DDesc &dd = c->h_ddesc[desc_off + d];
                const bool last = j + 1 == ch.steps;
                dd.Wp = nullptr; dd.blob = (const unsigned char *)ch.blobs[j]; dd.blob_bytes = ch.blob_bytes[j]; dd.n = ch.n;
                dd.W_out = nullptr; dd.m_out = last ? ch.m_out : nullptr; dd.v_out = last ? ch.v_out : nullptr;
                dd.cw = dd.cm = dd.cv = dd.head = nullptr; dd.wtype = (ch.flags >> 4) & 3u; dd.pad = 0;
                dd.tile_begin = dtile; dd.tile_count = tiles;
                c->h_tile_begin[g.tb_desc + d] = dtile;
                dtile += tiles;
            }
        }
        c->h_tile_begin[g.tb_desc + g.ndescs] = dtile;
        c->h_tile_begin[g.tb_chain + g.count] = ctile;
        tb_off += g.ndescs + g.count + 2;
        desc_off += g.ndescs;
        groups.push_back(g);
    }
    hipStream_t s = c->stream;
    if (count) {
        if (hipMemcpyAsync(c->ddesc_all, c->h_ddesc, sizeof(DDesc) * desc_off, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(c->cdesc_all, c->h_cdesc, sizeof(CDesc) * count, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(c->tile_begin_all, c->h_tile_begin, sizeof(u32) * tb_off, hipMemcpyHostToDevice, s) != hipSuccess)
            return enqueue_failed(c);
    }
    for (const CGroup &g : groups) {
        Workspace w = c->w;
        w.ddesc = c->ddesc_all + g.first_desc;
        w.dst = c->dst_all + g.first_desc;
        w.tile_begin = c->tile_begin_all + g.tb_desc;
        w.cdesc = c->cdesc_all + g.first;
        w.chain_tile_begin = c->tile_begin_all + g.tb_chain;
        w.rec_dev = c->w.rec_dev + g.first;
        w.rec_base = 0;
        const u32 dtiles = c->h_tile_begin[g.tb_desc + g.ndescs];
        bool moments = false;
        for (u32 q = 0; q < g.count; ++q)
            moments = moments || chains[g.first + q].m_out != nullptr || chains[g.first + q].v_out != nullptr;
        { StageTimer t(c, ST_MISC); launch_decode_parse(w, g.ndescs, false, s); }
        {
            StageTimer t(c, ST_DECODE_PREP);
            launch_decode_count(w, g.ndescs, dtiles, 0, s);
            launch_decode_scan(w, g.ndescs, 0, s);
            if (moments) { launch_decode_count(w, g.ndescs, dtiles, 1, s); launch_decode_scan(w, g.ndescs, 1, s); }
        }
        { StageTimer t(c, ST_DECODE_MAIN); launch_decode_chain(w, g.count, g.ntiles, s); }
        if (moments) {      // the last checkpoints' moments
            StageTimer t(c, ST_DECODE_MAIN);
            launch_decode_main(w, g.ndescs, dtiles, true, s);
            launch_decode_main16(w, g.ndescs, dtiles, true, s);
        }
        { StageTimer t(c, ST_MISC); launch_chain_finish(w, g.count, s); }
    }
    if (count) {
        if (hipMemcpyAsync(c->h_rec, c->w.rec_dev, sizeof(HostRec) * count, hipMemcpyDeviceToHost, s) != hipSuccess)
            return enqueue_failed(c);
    }
    if (hipMemcpyAsync(c->h_err, c->w.err_flag, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess) return enqueue_failed(c);
    if (hipGetLastError() != hipSuccess) return enqueue_failed(c);
    c->pending = 2;
    c->pending_count = count;
    return EXCP_OK;
}

int excp_collect(excp_ctx *c, excp_stats *stats) {
    if (!c) return EXCP_E_ARG;
    if (!c->pending) return EXCP_E_STATE;
    if (hipSetDevice(c->device) != hipSuccess) return EXCP_E_HIP;
    hipError_t e = hipStreamSynchronize(c->stream);
    c->pending = 0;
    for (int i = 0; i < ST_COUNT; ++i) { c->stage_ms[i] = 0; c->stage_launches[i] = 0; }
    for (auto &sp : c->spans) {
        float ms = 0.f;
        if (e == hipSuccess && hipEventElapsedTime(&ms, sp.a, sp.b) == hipSuccess) {
            c->stage_ms[sp.stage] += ms;
            c->stage_launches[sp.stage] += 1;
        }
        c->free_events.push_back(sp.a);
        c->free_events.push_back(sp.b);
    }
    c->spans.clear();
    if (e != hipSuccess) return EXCP_E_HIP;
    int first = EXCP_OK;
    if (*c->h_err) {
        first = EXCP_E_INTERNAL;
        launch_zero_u32((u32 *)c->w.err_flag, 4, c->stream);
        (void)hipStreamSynchronize(c->stream);
    }
    for (int i = 0; i < c->pending_count; ++i) {
        const HostRec &r = c->h_rec[i];
        if (stats) {
            excp_stats &o = stats[i];
            memset(&o, 0, sizeof(o));
            o.n = r.n; o.n_w = r.n_w; o.n_o = r.n_o; o.blob_bytes = r.blob_bytes; o.nonfinite = r.nonfinite;
            o.abs_sum_m = r.abs_sum; o.obj_w = r.obj[0]; o.obj_m = r.obj[1]; o.obj_v = r.obj[2];
            o.median_abs_dw = r.med; o.mean_abs_m = r.mean32; o.t_w = r.t_w; o.r_o = r.r_o;
            o.status = r.status;
        }
        if (first == EXCP_OK && r.status != 0) first = r.status;
    }
    return first;
}

int excp_compress_step(excp_ctx *c, const void *W_prev_recon, const void *W_t, const float *m_t,
                       const float *v_t, uint64_t n, float alpha, float beta, int nbits, int lloyd_iters,
                       uint32_t flags, void *blob_out, uint64_t blob_cap, uint64_t *blob_bytes,
                       void *W_recon_out, excp_stats *stats) {
    excp_tensor t{W_prev_recon, W_t, m_t, v_t, n, blob_out, blob_cap, W_recon_out};
    int rc = excp_compress_tensors(c, 1, &t, alpha, beta, nbits, lloyd_iters, flags);
    if (rc != EXCP_OK) return rc;
    excp_stats st;
    memset(&st, 0, sizeof(st));
    rc = excp_collect(c, &st);
    if (rc == EXCP_E_HIP || rc == EXCP_E_STATE) return rc;      // nothing was collected: the outputs stay untouched
    if (blob_bytes) *blob_bytes = st.blob_bytes;
    if (stats) *stats = st;
    return rc;
}

int excp_decompress_step(excp_ctx *c, const void *W_prev_recon, const void *blob, uint64_t blob_bytes,
                         uint64_t n, void *W_recon_out, float *m_out, float *v_out, uint32_t flags) {
    excp_blob b{W_prev_recon, blob, blob_bytes, n, W_recon_out, m_out, v_out, flags, 0};
    int rc = excp_decompress_tensors(c, 1, &b);
    if (rc != EXCP_OK) return rc;
    return excp_collect(c, nullptr);
}

int excp_decompress_step_static(int hip_device, void *hip_stream, const void *W_prev_recon, const void *blob,
                                uint64_t blob_bytes, uint64_t n, void *W_recon_out, float *m_out, float *v_out,
                                uint32_t flags) {
    if ((flags & ~0x30u) || (flags & 0x30u) == 0x30u) return EXCP_E_ARG;
    if (n > EXCP_STATIC_MAX_ELEMS) return EXCP_E_ARG;           // the static tables hold no more tiles than that
    if (!blob || ((uintptr_t)blob & 15u) || (n && !W_prev_recon)) return EXCP_E_ARG;
    if (hip_device < 0 || hip_device >= kMaxDevices) return EXCP_E_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || hip_device >= ndev) return EXCP_E_HIP;
    if (hipSetDevice(hip_device) != hipSuccess) return EXCP_E_HIP;
    StaticDevice sd;
    int rc = static_device(hip_device, sd);
    if (rc != EXCP_OK) return rc;
    hipStream_t s = (hipStream_t)hip_stream;

    Workspace w{};
    w.ddesc = (DDesc *)(sd.ptr + StaticOffsets::ddesc);
    w.dst = (DState *)(sd.ptr + StaticOffsets::dst);
    w.tile_begin = (u32 *)(sd.ptr + StaticOffsets::tile_begin);
    w.dec_kinds = (u32 *)(sd.ptr + StaticOffsets::dec_kinds);
    w.rec_dev = (HostRec *)(sd.ptr + StaticOffsets::rec);
    w.dec_part = (u64 *)(sd.ptr + StaticOffsets::dec_part);
    w.dec_cnt_w = (u32 *)(sd.ptr + StaticOffsets::cnt_w);
    w.dec_cnt_o = (u32 *)(sd.ptr + StaticOffsets::cnt_o);
    w.rec_base = 0;
    w.cus = sd.cus;

    DDesc d{};
    d.Wp = (const float *)W_prev_recon; d.blob = (const unsigned char *)blob; d.blob_bytes = blob_bytes; d.n = n;
    d.W_out = (float *)W_recon_out; d.m_out = m_out; d.v_out = v_out;
    d.cw = d.cm = d.cv = d.head = nullptr; d.wtype = (flags >> 4) & 3u; d.pad = 0;
    d.tile_begin = 0; d.tile_count = (u32)((n + EXCP_TILE - 1) / EXCP_TILE);
    const u32 ntiles = d.tile_count;
    const bool moments = m_out != nullptr || v_out != nullptr;

    // Nothing of the previous call is relied on: the descriptor, the tile table and the kinds word are
    // written first, the state and every count of the tiles in use are written by the kernels before
    // they are read, and the record is written last.
    launch_decode_single_setup(w, d, s);
    launch_decode_parse(w, 1, true, s);
    launch_decode_count(w, 1, ntiles, 0, s);
    launch_decode_scan(w, 1, 0, s);
    if (moments) {
        launch_decode_count(w, 1, ntiles, 1, s);
        launch_decode_scan(w, 1, 1, s);
    }
    launch_decode_main(w, 1, ntiles, moments, s);
    launch_decode_main16(w, 1, ntiles, moments, s);
    launch_decode_raw(w, 1, ntiles, moments, s);
    launch_decode_finish(w, 1, s);
    if (hipGetLastError() != hipSuccess) { (void)hipStreamSynchronize(s); return EXCP_E_HIP; }
    HostRec rec;
    memset(&rec, 0, sizeof(rec));
    if (hipMemcpyAsync(&rec, w.rec_dev, sizeof(HostRec), hipMemcpyDeviceToHost, s) != hipSuccess) {
        (void)hipStreamSynchronize(s);
        return EXCP_E_HIP;
    }
    if (hipStreamSynchronize(s) != hipSuccess) return EXCP_E_HIP;
    return rec.status;
}

}  // extern "C"
