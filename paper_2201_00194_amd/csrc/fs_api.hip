// Host side of the C ABI: argument validation, model packing, descriptor upload, launches.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "fs_internal.h"

namespace fs {

// ---- errors ------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int fail_hip(hipError_t e, const char *what)
{
    (void)hipGetLastError();  // clear the sticky launch error, the code is reported here
    if (e == hipErrorOutOfMemory)
        return fail(FS_ENOMEM, "%s: %s", what, hipGetErrorString(e));
    return fail(FS_EDEVICE, "%s: %s", what, hipGetErrorString(e));
}

// ---- per-device state: descriptor ring and scratch ---------------------------------------------
constexpr int kSlots = 8;
constexpr int kMaxDevices = 16;
constexpr size_t kSlotBytes = 65536;   // descriptor staging a slot starts with

struct Slot {
    void *d_buf = nullptr;
    void *h_buf = nullptr;  // pinned
    size_t cap = 0;
    hipEvent_t done = nullptr;
    bool used = false;
};

// Two scratch regions per device, so that a scoring call and a top-k call never share bytes.
enum { kScratchScore = 0, kScratchTopk = 1, kScratchRegions = 2 };

// Descriptors of up to kInlineBytes travel as kernel arguments: a small kernel stores them into
// a fixed device buffer (one per kind of call), in stream order in front of the kernels that read
// them.  No pinned staging, no copy, no event and nothing to wait for, so such a call can also be
// recorded into a HIP graph.  Longer descriptor arrays go through the ring of pinned slots.
constexpr size_t kInlineBytes = 16384;
constexpr size_t kBlobBytes = 3968;               // one kernel argument (the limit is 4 KB)
enum { kDescScore = 0, kDescTopk = 1, kDescKinds = 2 };

struct DeviceCtx {
    Slot slots[kSlots];
    int next = 0;
    float *scratch[kScratchRegions] = {nullptr, nullptr};
    size_t scratch_floats[kScratchRegions] = {0, 0};
    void *inline_dev[kDescKinds] = {nullptr, nullptr};
    void *inline_host[kDescKinds] = {nullptr, nullptr};
    int n_compute_units = 0;
};

struct DescBlob {
    uint32_t words[kBlobBytes / 4];
};

__global__ void __launch_bounds__(256) desc_store_kernel(DescBlob blob, uint32_t *dst, int n_words)
{
    for (int i = threadIdx.x; i < n_words; i += blockDim.x)
        dst[i] = blob.words[i];
}

// Where a call builds its descriptors (host) and where the kernels read them (dev).
struct DescBuf {
    void *host = nullptr;
    void *dev = nullptr;
    Slot *slot = nullptr;                          // null: the inline path
};

static std::mutex g_mu;
static DeviceCtx g_ctx[kMaxDevices];

static int current_ctx(DeviceCtx **out, int *dev_out = nullptr)
{
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(FS_EUNSUPPORTED, "device ordinal %d not supported", dev);
    *out = &g_ctx[dev];
    if (g_ctx[dev].n_compute_units == 0) {
        int n = 0;
        FS_HIP(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
        g_ctx[dev].n_compute_units = n > 0 ? n : 256;
    }
    if (dev_out)
        *dev_out = dev;
    return FS_OK;
}

// A slot whose previous use has finished, with room for `bytes`.
static int acquire_slot(DeviceCtx *ctx, size_t bytes, Slot **out)
{
    Slot *s = &ctx->slots[ctx->next];
    ctx->next = (ctx->next + 1) % kSlots;
    if (!s->done)
        FS_HIP(hipEventCreateWithFlags(&s->done, hipEventDisableTiming));
    if (s->used)
        FS_HIP(hipEventSynchronize(s->done));
    if (s->cap < bytes) {
        size_t cap = bytes < kSlotBytes ? kSlotBytes : bytes * 2;
        if (s->d_buf)
            FS_HIP(hipFree(s->d_buf));
        if (s->h_buf)
            FS_HIP(hipHostFree(s->h_buf));
        s->d_buf = s->h_buf = nullptr;
        s->cap = 0;
        FS_HIP(hipMalloc(&s->d_buf, cap));
        FS_HIP(hipHostMalloc(&s->h_buf, cap, hipHostMallocDefault));
        s->cap = cap;
    }
    *out = s;
    return FS_OK;
}

// Region `which` with room for `floats`; `exact` reserves just that (fs_workspace_reserve),
// otherwise a quarter more so that slowly growing calls do not re-allocate every time.
static int ensure_scratch(DeviceCtx *ctx, int which, size_t floats, bool exact = false)
{
    if (ctx->scratch_floats[which] >= floats)
        return FS_OK;
    // Earlier submissions may still read the old buffer.
    FS_HIP(hipDeviceSynchronize());
    if (ctx->scratch[which])
        FS_HIP(hipFree(ctx->scratch[which]));
    ctx->scratch[which] = nullptr;
    ctx->scratch_floats[which] = 0;
    size_t want = exact ? floats : floats + floats / 4 + 1024;
    FS_HIP(hipMalloc((void **)&ctx->scratch[which], want * sizeof(float)));
    ctx->scratch_floats[which] = want;
    return FS_OK;
}

static int ensure_inline(DeviceCtx *ctx, int kind)
{
    if (!ctx->inline_dev[kind])
        FS_HIP(hipMalloc(&ctx->inline_dev[kind], kInlineBytes));
    if (!ctx->inline_host[kind]) {
        ctx->inline_host[kind] = malloc(kInlineBytes);
        if (!ctx->inline_host[kind])
            return fail(FS_ENOMEM, "host allocation failed");
    }
    return FS_OK;
}

static int acquire_desc(DeviceCtx *ctx, int kind, size_t bytes, DescBuf *out)
{
    *out = DescBuf();
    if (bytes <= kInlineBytes) {
        int rc = ensure_inline(ctx, kind);
        if (rc != FS_OK)
            return rc;
        out->host = ctx->inline_host[kind];
        out->dev = ctx->inline_dev[kind];
        return FS_OK;
    }
    int rc = acquire_slot(ctx, bytes, &out->slot);
    if (rc != FS_OK)
        return rc;
    out->host = out->slot->h_buf;
    out->dev = out->slot->d_buf;
    return FS_OK;
}

// Descriptors to the device, in stream order in front of the kernels that follow.
static int commit_desc(const DescBuf &db, size_t bytes, hipStream_t stream)
{
    if (db.slot) {
        FS_HIP(hipMemcpyAsync(db.dev, db.host, bytes, hipMemcpyHostToDevice, stream));
        db.slot->used = true;
        return FS_OK;
    }
    for (size_t at = 0; at < bytes; at += kBlobBytes) {
        const size_t n = bytes - at < kBlobBytes ? bytes - at : kBlobBytes;
        DescBlob blob;
        memcpy(blob.words, (const char *)db.host + at, n);
        hipLaunchKernelGGL(desc_store_kernel, dim3(1), dim3(256), 0, stream, blob,
                           (uint32_t *)((char *)db.dev + at), (int)((n + 3) / 4));
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return fail_hip(e, "desc_store_kernel launch");
    }
    return FS_OK;
}

// After the last kernel of the call: the slot may be reused once this point is reached.
static int finish_desc(const DescBuf &db, hipStream_t stream)
{
    if (db.slot)
        FS_HIP(hipEventRecord(db.slot->done, stream));
    return FS_OK;
}

// ---- test and tuning overrides -----------------------------------------------------------------
static std::mutex g_tune_mu;
static int g_tune[FS_TUNE_OPTIONS] = {-1, -1, -1, -1, -1, -1, -1, -1, -1};

int tune(int option)
{
    std::lock_guard<std::mutex> lock(g_tune_mu);
    return option >= 0 && option < FS_TUNE_OPTIONS ? g_tune[option] : -1;
}

// ---- optional per-kernel timing -------------------------------------------------------------
struct ProfRecord {
    hipEvent_t a, b;
    int kernel_class;
};
static std::mutex g_prof_mu;
static std::vector<ProfRecord> g_prof;
static size_t g_prof_used = 0;
static bool g_prof_on = false;
static bool g_prof_open = false;

void prof_start(int kernel_class, hipStream_t stream)
{
    std::lock_guard<std::mutex> lock(g_prof_mu);
    g_prof_open = false;
    if (!g_prof_on || g_prof_used >= g_prof.size())
        return;
    ProfRecord &r = g_prof[g_prof_used];
    r.kernel_class = kernel_class;
    if (hipEventRecord(r.a, stream) == hipSuccess)
        g_prof_open = true;
}

void prof_stop(hipStream_t stream)
{
    std::lock_guard<std::mutex> lock(g_prof_mu);
    if (!g_prof_open)
        return;
    g_prof_open = false;
    if (hipEventRecord(g_prof[g_prof_used].b, stream) == hipSuccess)
        ++g_prof_used;
}

}  // namespace fs

using namespace fs;

extern "C" int fs_profile_begin(int32_t max_records)
{
    std::lock_guard<std::mutex> lock(g_prof_mu);
    if (max_records < 1 || max_records > (1 << 20))
        return fail(FS_EINVAL, "fs_profile_begin: max_records %d outside [1, 2^20]", max_records);
    g_prof_on = false;
    g_prof_used = 0;
    while (g_prof.size() < (size_t)max_records) {
        ProfRecord r;
        r.kernel_class = 0;
        FS_HIP(hipEventCreate(&r.a));
        hipError_t e = hipEventCreate(&r.b);
        if (e != hipSuccess) {
            (void)hipEventDestroy(r.a);
            return fail_hip(e, "hipEventCreate");
        }
        try {
            g_prof.push_back(r);
        } catch (const std::bad_alloc &) {
            (void)hipEventDestroy(r.a);
            (void)hipEventDestroy(r.b);
            return fail(FS_ENOMEM, "fs_profile_begin: host allocation failed");
        }
    }
    g_prof_on = true;
    return FS_OK;
}

extern "C" int fs_profile_end(double *ms_by_kernel, int32_t *launches_by_kernel)
{
    std::lock_guard<std::mutex> lock(g_prof_mu);
    g_prof_on = false;
    for (int c = 0; c < kKernClasses; ++c) {
        if (ms_by_kernel) ms_by_kernel[c] = 0.0;
        if (launches_by_kernel) launches_by_kernel[c] = 0;
    }
    for (size_t i = 0; i < g_prof_used; ++i) {
        FS_HIP(hipEventSynchronize(g_prof[i].b));
        float ms = 0.f;
        FS_HIP(hipEventElapsedTime(&ms, g_prof[i].a, g_prof[i].b));
        const int c = g_prof[i].kernel_class;
        if (ms_by_kernel) ms_by_kernel[c] += ms;
        if (launches_by_kernel) launches_by_kernel[c] += 1;
    }
    g_prof_used = 0;
    return FS_OK;
}

// ---- small entry points ------------------------------------------------------------------------
extern "C" const char *fs_last_error(void) { return fs::g_err; }
extern "C" int fs_version(void) { return 200; }

extern "C" int fs_tune_set(int32_t option, int32_t value)
{
    if (option < 0 || option >= FS_TUNE_OPTIONS)
        return fail(FS_EINVAL, "fs_tune_set: unknown option %d", option);
    std::lock_guard<std::mutex> lock(g_tune_mu);
    g_tune[option] = value < 0 ? -1 : value;
    return FS_OK;
}

extern "C" int32_t fs_tune_get(int32_t option) { return tune(option); }

extern "C" int64_t fs_colblock64_floats(int64_t n_rows, int32_t n_features)
{
    if (n_rows < 0 || n_features < 0)
        return 0;
    return ((n_rows + 63) / 64) * 64 * (int64_t)n_features;
}

// ---- scoring -----------------------------------------------------------------------------------
// Tile groups one workgroup of the LDS traversal takes in a row.  From the second group on, a
// group's tiles are fetched while the one before it is still being walked, which hides about
// 1 us of fetch latency per group; the price is a coarser tail at the end of the launch, half a
// workgroup's time on average.  With R rounds of groups per compute unit and t us per group,
// G groups per workgroup save R (1 - 1/G) us and cost G t / 2 us: best at G = sqrt(2 R / t).
// Measured (traversal of configs[3] at full / half / quarter size, configs[4], the foresee
// step; best G and what it gains): 4 (-3.3 %), 4-6 (-1.6 %), 2-3 (-0.7 %), 1 (any G > 1 loses,
// 51 us per group), 6 (-2.6 %; 4: -1.8 %).
constexpr int kLdsMaxGroupsPerWg = 4;

static int lds_groups_wanted(int64_t groups_in_launch, double group_us, int n_compute_units)
{
    const int forced = tune(FS_TUNE_LDS_GROUPS);
    if (forced >= 1)
        return forced > 16 ? 16 : forced;
    if (groups_in_launch <= 0 || group_us <= 0.0)
        return 1;
    const double rounds = (double)groups_in_launch / (double)n_compute_units;
    int g = (int)sqrt(2.0 * rounds / group_us);
    if (g < 1) g = 1;
    if (g > kLdsMaxGroupsPerWg) g = kLdsMaxGroupsPerWg;
    return g;
}

// Row-major input needs no pass of its own where the first kernel to touch the features can
// read it: the rank-coding kernel always can; the LDS kernel transposes tiles on their way
// into LDS (through the still unused chunk region) when rows are whole 16-byte pieces and at
// least 8 padded rows fit below the tiles.  Other row-major families are re-tiled into scratch.
static bool rowmajor_in_kernel(const fs_model *m)
{
    if (m->rank_ok)
        return true;
    return m->lds_ok && m->n_features % 4 == 0 && m->lds_tile0 >= 8 * (m->n_features + 1) * 4;
}

// Validates the family descriptors (everything that does not need the device) and adds up the
// scoring scratch the call uses, in floats.  `dev` < 0: the models' device is not checked.
static int score_scratch_floats(const char *who, int32_t n_families, const fs_family *fams, int dev,
                                size_t *out)
{
    size_t scratch_floats = 0;
    for (int f = 0; f < n_families; ++f) {
        const fs_family &a = fams[f];
        if (!a.model)
            return fail(FS_EINVAL, "%s: family %d has no model", who, f);
        if (dev >= 0 && a.model->device != dev)
            return fail(FS_EINVAL, "%s: family %d: model lives on device %d, "
                        "current device is %d", who, f, a.model->device, dev);
        if (a.n_rows < 0 || a.n_rows >= ((int64_t)1 << 31))
            return fail(FS_EINVAL, "%s: family %d: n_rows %lld outside [0, 2^31)", who, f,
                        (long long)a.n_rows);
        if (a.n_programs < 0)
            return fail(FS_EINVAL, "%s: family %d: n_programs is negative", who, f);
        if (a.layout != FS_ROWMAJOR && a.layout != FS_COLBLOCK64)
            return fail(FS_EINVAL, "%s: family %d: unknown layout %d", who, f, a.layout);
        if (a.n_rows > 0 && !a.features)
            return fail(FS_EINVAL, "%s: family %d: features is NULL", who, f);
        if (((uintptr_t)a.features & 15) != 0)
            return fail(FS_EINVAL, "%s: family %d: features not 16-byte aligned", who, f);
        if (a.n_programs > 0 && !a.prog_off)
            return fail(FS_EINVAL, "%s: family %d: prog_off is NULL", who, f);
        if (a.n_programs > 0 && !a.prog_score)
            return fail(FS_EINVAL, "%s: family %d: prog_score is NULL", who, f);
        if (a.n_programs == 0 && a.n_rows != 0)
            return fail(FS_EINVAL, "%s: family %d: %lld rows but no programs", who, f,
                        (long long)a.n_rows);
        if (!a.row_score)
            scratch_floats += (size_t)a.n_rows;
        if (a.model->rank_ok)                                // u16 rank tiles, in float units
            scratch_floats += (size_t)((a.n_rows + 63) / 64) * 32 * (size_t)rank_tile_cols(a.model->n_features) + 4;
        if ((a.model->rank_ok || a.model->lds_ok) && a.layout == FS_ROWMAJOR &&
            !rowmajor_in_kernel(a.model))                                         // re-tiled copy
            scratch_floats += (size_t)((a.n_rows + 63) / 64) * 64 * (size_t)a.model->n_features + 4;
    }
    *out = scratch_floats;
    return FS_OK;
}

extern "C" size_t fs_workspace_bytes(int32_t n_families, const fs_family *fams)
{
    if (n_families <= 0 || !fams) {
        if (n_families < 0 || (n_families > 0 && !fams))
            (void)fail(FS_EINVAL, "fs_workspace_bytes: bad arguments");
        return 0;
    }
    size_t floats = 0;
    if (score_scratch_floats("fs_workspace_bytes", n_families, fams, -1, &floats) != FS_OK)
        return 0;
    return floats * sizeof(float);
}

extern "C" int fs_workspace_reserve(size_t score_bytes, size_t topk_bytes)
{
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceCtx *ctx = nullptr;
    int rc = current_ctx(&ctx);
    if (rc != FS_OK)
        return rc;
    rc = ensure_scratch(ctx, kScratchScore, (score_bytes + 3) / 4, true);
    if (rc == FS_OK)
        rc = ensure_scratch(ctx, kScratchTopk, (topk_bytes + 3) / 4, true);
    for (int kind = 0; kind < kDescKinds && rc == FS_OK; ++kind)
        rc = ensure_inline(ctx, kind);
    for (int i = 0; i < kSlots && rc == FS_OK; ++i) {       // staging of every slot of the ring
        Slot *s = &ctx->slots[i];
        if (!s->done)
            FS_HIP(hipEventCreateWithFlags(&s->done, hipEventDisableTiming));
        if (s->cap == 0) {
            FS_HIP(hipMalloc(&s->d_buf, kSlotBytes));
            FS_HIP(hipHostMalloc(&s->h_buf, kSlotBytes, hipHostMallocDefault));
            s->cap = kSlotBytes;
        }
    }
    return rc;
}

extern "C" int fs_score_families(int32_t n_families, const fs_family *fams, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (n_families < 0)
        return fail(FS_EINVAL, "fs_score_families: n_families %d is negative", n_families);
    if (n_families == 0)
        return FS_OK;
    if (!fams)
        return fail(FS_EINVAL, "fs_score_families: fams is NULL");

    std::lock_guard<std::mutex> lock(g_mu);
    DeviceCtx *ctx = nullptr;
    int dev = 0;
    int rc = current_ctx(&ctx, &dev);
    if (rc != FS_OK)
        return rc;

    size_t scratch_floats = 0;
    rc = score_scratch_floats("fs_score_families", n_families, fams, dev, &scratch_floats);
    if (rc != FS_OK)
        return rc;
    rc = ensure_scratch(ctx, kScratchScore, scratch_floats);
    if (rc != FS_OK)
        return rc;

    DescBuf db;
    rc = acquire_desc(ctx, kDescScore, sizeof(FamDesc) * (size_t)n_families, &db);
    if (rc != FS_OK)
        return rc;
    FamDesc *h = (FamDesc *)db.host;
    int64_t trav_blocks = 0, seg_blocks = 0, lds_blocks[kLdsModes] = {0, 0};
    int64_t rk_blocks = 0, bin_blocks = 0, retile_blocks = 0;
    bool rk_dump = false;
    bool dump[kLdsModes] = {false, false};
    // tile groups the LDS kernel will see, per workgroup shape (row-major families included:
    // they count towards the length of the launch, though their workgroups take one group each)
    int64_t lds_groups[kLdsModes] = {0, 0};
    double lds_us[kLdsModes] = {0.0, 0.0};           // all groups of the launch, by the planner's estimate
    for (int f = 0; f < n_families; ++f) {
        const fs_model *m = fams[f].model;
        if (!m->rank_ok && m->lds_ok) {
            const int64_t g = ((fams[f].n_rows + 63) / 64 + m->lds_tiles - 1) / m->lds_tiles;
            lds_groups[m->lds_mode] += g;
            lds_us[m->lds_mode] += (double)g * (double)m->lds_group_us;
        }
    }
    int groups_per_wg[kLdsModes];
    for (int md = 0; md < kLdsModes; ++md) {
        const double group_us = lds_groups[md] ? lds_us[md] / (double)lds_groups[md] : 0.0;
        groups_per_wg[md] = lds_groups_wanted(lds_groups[md], group_us, ctx->n_compute_units);
        if (tune(FS_TUNE_VERBOSE) > 0 && lds_groups[md] > 0)
            fprintf(stderr, "fs_score_families: %lld tile groups of about %.1f us, LDS shape %d: %d per workgroup\n",
                    (long long)lds_groups[md], group_us, md, groups_per_wg[md]);
    }
    size_t scratch_pos = 0;
    for (int f = 0; f < n_families; ++f) {
        const fs_family &a = fams[f];
        FamDesc d;
        d.nodes = a.model->d_nodes;
        d.tree_off = a.model->d_tree_off;
        d.features = a.features;
        d.prog_off = a.prog_off;
        d.prog_score = a.prog_score;
        if (a.row_score) {
            d.row_score = a.row_score;
        } else {
            d.row_score = ctx->scratch[kScratchScore] + scratch_pos;
            scratch_pos += (size_t)a.n_rows;
        }
        d.leaf_idx = a.leaf_idx;
        d.n_trees = a.model->n_trees;
        d.n_features = a.model->n_features;
        d.layout = a.layout;
        d.n_rows = (int32_t)a.n_rows;
        d.n_programs = a.n_programs;
        d.bias = a.model->bias;
        d.trav_block0 = (int32_t)trav_blocks;
        d.seg_block0 = (int32_t)seg_blocks;
        for (int md = 0; md < kLdsModes; ++md)
            d.lds_block0[md] = (int32_t)lds_blocks[md];
        d.image = a.model->d_image;
        d.chunks = a.model->d_chunks;
        d.slot_ids = a.model->d_slot_ids;
        d.n_chunks = a.model->n_chunks;
        d.lds_tile0 = a.model->lds_tile0;
        d.lds_tiles = a.model->lds_tiles;
        d.compact = a.model->compact ? 1 : 0;
        // Row-major features of a model that has an LDS format: transposed inside the LDS kernel
        // where that is possible, else re-tiled into scratch first (one extra pass over the
        // features; from then on the family is column-blocked).
        d.rowmajor_src = nullptr;
        d.retile_block0 = (int32_t)retile_blocks;
        d.retile_colblocks = 0;
        const bool fast = a.model->rank_ok || a.model->lds_ok;
        const bool in_kernel = a.layout == FS_ROWMAJOR && rowmajor_in_kernel(a.model);
        if (fast && a.layout == FS_ROWMAJOR && a.n_rows > 0 && !in_kernel) {
            const int64_t tiles = (a.n_rows + 63) / 64;
            scratch_pos = (scratch_pos + 3) & ~(size_t)3;
            d.rowmajor_src = a.features;
            d.features = ctx->scratch[kScratchScore] + scratch_pos;
            d.layout = FS_COLBLOCK64;
            scratch_pos += (size_t)tiles * 64 * (size_t)a.model->n_features;
            d.retile_colblocks = (a.model->n_features + 127) / 128;
            retile_blocks += tiles * d.retile_colblocks;
        }
        const bool colblock = d.layout == FS_COLBLOCK64;
        d.rk_nodes = a.model->d_rk_nodes;
        d.rk_ids = a.model->d_rk_ids;
        d.cuts = a.model->d_cuts;
        d.ranks = nullptr;
        d.rk_depth = a.model->rk_depth;
        d.rk_tiles = a.model->rk_tiles;
        d.rk_trees_per_chunk = a.model->rk_trees_per_chunk;
        d.rk_tree_bytes = a.model->rk_tree_bytes;
        d.rk_tile0 = a.model->rk_tile0;
        d.rk_block0 = (int32_t)rk_blocks;
        d.bin_block0 = (int32_t)bin_blocks;
        d.bin_groups = 1;
        d.bin_feats_per_group = a.model->n_features;
        d.bin_tiles_per_block = kBinTilesPerBlock;
        d.cut_bits = a.model->cut_bits;
        d.pad = 0;
        // Column-blocked features: deep perfect-tree models are rank-coded first and walked by
        // the rank kernel, other models that fit the LDS format take the LDS kernel; everything
        // else is walked from global memory.
        if (a.model->rank_ok && (colblock || in_kernel)) {
            const int64_t tiles = (a.n_rows + 63) / 64;
            scratch_pos = (scratch_pos + 3) & ~(size_t)3;            // 16-byte aligned tiles
            d.ranks = (uint16_t *)(ctx->scratch[kScratchScore] + scratch_pos);
            scratch_pos += (size_t)tiles * 32 * (size_t)rank_tile_cols(a.model->n_features);
            const int len = 1 << a.model->cut_bits;
            int per_group = kBinTableBytes / 4 / len;
            if (per_group > a.model->n_features) per_group = a.model->n_features;
            d.bin_feats_per_group = per_group;                      // >= 1 by model packing
            d.bin_groups = (a.model->n_features + per_group - 1) / per_group;
            // enough workgroups to fill the chip even for a small family
            int64_t tpb = tiles * d.bin_groups / 512;
            if (tpb < 8) tpb = 8;
            if (tpb > kBinTilesPerBlock) tpb = kBinTilesPerBlock;
            d.bin_tiles_per_block = (int32_t)tpb;
            bin_blocks += (int64_t)d.bin_groups * ((tiles + tpb - 1) / tpb);
            rk_blocks += (tiles + a.model->rk_tiles - 1) / a.model->rk_tiles;
            if (a.leaf_idx && a.n_rows > 0)
                rk_dump = true;
        } else if (a.model->lds_ok && (colblock || in_kernel)) {
            const int64_t tiles = (a.n_rows + 63) / 64;
            const int md = a.model->lds_mode;
            const int64_t groups = (tiles + a.model->lds_tiles - 1) / a.model->lds_tiles;
            const int per_wg = lds_groups_per_wg(d.layout, a.model->n_features, a.model->lds_tiles,
                                                 64 * kLdsModeWaves[md], groups_per_wg[md]);
            lds_blocks[md] += (groups + per_wg - 1) / per_wg;
            if (a.leaf_idx && a.n_rows > 0)
                dump[md] = true;
        } else
        trav_blocks += (a.n_rows + kTravRowsPerBlock - 1) / kTravRowsPerBlock;
        seg_blocks += (a.n_programs + kSegProgsPerBlock - 1) / kSegProgsPerBlock;
        h[f] = d;
    }
    if (trav_blocks >= ((int64_t)1 << 31) || seg_blocks >= ((int64_t)1 << 31) ||
        lds_blocks[0] >= ((int64_t)1 << 31) || lds_blocks[1] >= ((int64_t)1 << 31) ||
        rk_blocks >= ((int64_t)1 << 31) || bin_blocks >= ((int64_t)1 << 31) ||
        retile_blocks >= ((int64_t)1 << 31))
        return fail(FS_EUNSUPPORTED, "fs_score_families: too much work for one submission");

    rc = commit_desc(db, sizeof(FamDesc) * (size_t)n_families, stream);
    if (rc != FS_OK)
        return rc;
    const FamDesc *d_desc = (const FamDesc *)db.dev;
    if (retile_blocks > 0) {
        prof_start(kKernPack, stream);
        rc = launch_retile(d_desc, n_families, (int)retile_blocks, stream);
        prof_stop(stream);
    }
    for (int md = 0; md < kLdsModes && rc == FS_OK; ++md) {
        if (lds_blocks[md] == 0)
            continue;
        prof_start(kKernTraverse, stream);
        rc = launch_traverse_lds(d_desc, n_families, md, (int)lds_blocks[md], groups_per_wg[md],
                                 dump[md], stream);
        prof_stop(stream);
    }
    if (rc == FS_OK && bin_blocks > 0) {
        prof_start(kKernRankCode, stream);
        rc = launch_rank_code(d_desc, n_families, (int)bin_blocks, stream);
        prof_stop(stream);
    }
    if (rc == FS_OK && rk_blocks > 0) {
        prof_start(kKernTraverseRank, stream);
        rc = launch_traverse_rank(d_desc, n_families, (int)rk_blocks, rk_dump, stream);
        prof_stop(stream);
    }
    if (rc == FS_OK && trav_blocks > 0) {
        prof_start(kKernTraverseGlobal, stream);
        rc = launch_traverse_global(d_desc, n_families, (int)trav_blocks, stream);
        prof_stop(stream);
    }
    if (rc == FS_OK && seg_blocks > 0) {
        prof_start(kKernSegsum, stream);
        rc = launch_segsum(d_desc, n_families, (int)seg_blocks, stream);
        prof_stop(stream);
    }
    const int rc2 = finish_desc(db, stream);
    return rc != FS_OK ? rc : rc2;
}

// ---- top-k -------------------------------------------------------------------------------------
struct TopkSizes {
    size_t n_blocks = 0, n_merge = 0, comp_total = 0, n_pairs_total = 0;
    int max_comp = 0, n_levels = 0, max_k = 0;
};

// Validates the requests and sizes the submission: first-stage workgroups, LDS merges, pairwise
// merges per level, scratch composites (8 bytes each).
static int topk_sizes(const char *who, int32_t n_requests, const fs_topk_req *reqs, TopkSizes *out)
{
    TopkSizes z;
    for (int i = 0; i < n_requests; ++i) {
        const fs_topk_req &r = reqs[i];
        if (r.n < 0 || r.k < 0)
            return fail(FS_EINVAL, "%s: request %d: n=%d k=%d must be non-negative", who, i, r.n, r.k);
        if (r.k > FS_MAX_TOPK)
            return fail(FS_EUNSUPPORTED, "%s: request %d: k=%d exceeds FS_MAX_TOPK=%d", who, i, r.k,
                        FS_MAX_TOPK);
        if (r.n > 0 && !r.score)
            return fail(FS_EINVAL, "%s: request %d: score is NULL", who, i);
        if (r.k > 0 && !r.out_idx)
            return fail(FS_EINVAL, "%s: request %d: out_idx is NULL", who, i);
        if (r.k > z.max_k)
            z.max_k = r.k;
    }
    for (int i = 0; i < n_requests; ++i) {
        const fs_topk_req &r = reqs[i];
        const TopkPlan p = topk_plan(r.n, r.k);
        z.n_blocks += (size_t)p.s;
        if (p.mode == 1) {
            ++z.n_merge;
            z.comp_total += (size_t)p.s * (size_t)r.k;
            int kp = 1;
            while (kp < r.k)
                kp <<= 1;
            if (p.s * kp > z.max_comp)
                z.max_comp = p.s * kp;
        } else if (p.mode == 2) {
            // first-stage lists: min(k, length) per slice
            const size_t every = (size_t)r.n, capped = (size_t)p.s * (size_t)r.k;
            z.comp_total += every < capped ? every : capped;
            int lists = p.s, levels = 0;
            while (lists > 1) {
                const int pairs = lists / 2;
                z.n_pairs_total += (size_t)pairs;
                if (lists > 2)
                    z.comp_total += (size_t)pairs * (size_t)r.k;   // merged lists (the last level writes the answer)
                lists = pairs + (lists & 1);
                ++levels;
            }
            if (levels > z.n_levels)
                z.n_levels = levels;
        }
    }
    *out = z;
    return FS_OK;
}

extern "C" size_t fs_topk_workspace_bytes(int32_t n_requests, const fs_topk_req *reqs)
{
    if (n_requests <= 0 || !reqs) {
        if (n_requests < 0 || (n_requests > 0 && !reqs))
            (void)fail(FS_EINVAL, "fs_topk_workspace_bytes: bad arguments");
        return 0;
    }
    TopkSizes z;
    if (topk_sizes("fs_topk_workspace_bytes", n_requests, reqs, &z) != FS_OK)
        return 0;
    return z.comp_total * sizeof(unsigned long long);
}

extern "C" int fs_topk(int32_t n_requests, const fs_topk_req *reqs, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (n_requests < 0)
        return fail(FS_EINVAL, "fs_topk: n_requests %d is negative", n_requests);
    if (n_requests == 0)
        return FS_OK;
    if (!reqs)
        return fail(FS_EINVAL, "fs_topk: reqs is NULL");
    TopkSizes z;
    int rc = topk_sizes("fs_topk", n_requests, reqs, &z);
    if (rc != FS_OK)
        return rc;
    const int max_k = z.max_k;
    if (max_k == 0)
        return FS_OK;

    std::lock_guard<std::mutex> lock(g_mu);
    DeviceCtx *ctx = nullptr;
    rc = current_ctx(&ctx);
    if (rc != FS_OK)
        return rc;
    auto plan_of = [](const fs_topk_req &r) { return topk_plan(r.n, r.k); };
    typedef TopkPlan Plan;
    const size_t n_blocks = z.n_blocks, n_merge = z.n_merge, comp_total = z.comp_total,
                 n_pairs_total = z.n_pairs_total;
    const int max_comp = z.max_comp, n_levels = z.n_levels;
    if (comp_total) {
        rc = ensure_scratch(ctx, kScratchTopk, comp_total * 2);
        if (rc != FS_OK)
            return rc;
    }
    const size_t desc_bytes = sizeof(TopkDesc) * n_blocks;
    const size_t merge_off = (desc_bytes + 15) & ~(size_t)15;
    const size_t path_off = (merge_off + sizeof(TopkMergeDesc) * n_merge + 15) & ~(size_t)15;
    const size_t total_bytes = path_off + sizeof(TopkPairDesc) * n_pairs_total;
    DescBuf db;
    rc = acquire_desc(ctx, kDescTopk, total_bytes, &db);
    if (rc != FS_OK)
        return rc;
    TopkDesc *h = (TopkDesc *)db.host;
    TopkMergeDesc *hm = (TopkMergeDesc *)((char *)db.host + merge_off);
    TopkPairDesc *hp = (TopkPairDesc *)((char *)db.host + path_off);
    unsigned long long *comp = (unsigned long long *)ctx->scratch[kScratchTopk];
    // merge-path descriptors are stored level by level: first count the pairs of every level
    constexpr int kMaxLevels = 8;
    size_t level_pairs[kMaxLevels] = {0}, level_at[kMaxLevels] = {0};
    int level_entries[kMaxLevels] = {0};        // longest la + lb of the level: sizes its grid
    for (int i = 0; i < n_requests; ++i) {
        const Plan p = plan_of(reqs[i]);
        if (p.mode != 2)
            continue;
        int lists = p.s, lv = 0;
        while (lists > 1) {
            level_pairs[lv++] += (size_t)(lists / 2);
            lists = lists / 2 + (lists & 1);
        }
    }
    for (int lv = 1; lv < kMaxLevels; ++lv)
        level_at[lv] = level_at[lv - 1] + level_pairs[lv - 1];
    size_t level_fill[kMaxLevels];
    for (int lv = 0; lv < kMaxLevels; ++lv)
        level_fill[lv] = level_at[lv];
    size_t b = 0, m = 0;
    for (int i = 0; i < n_requests; ++i) {
        const fs_topk_req &r = reqs[i];
        const Plan p = plan_of(r);
        // lists of a mode-2 request: pointer and length of every current list
        const unsigned long long *list_ptr[kTopkWideMaxSlices];
        int list_len[kTopkWideMaxSlices];
        unsigned long long *first = comp;
        for (int j = 0; j < p.s; ++j, ++b) {
            h[b].score = r.score;
            h[b].out_idx = r.out_idx;
            h[b].out_score = r.out_score;
            h[b].n = r.n;
            h[b].k = r.k;
            const long long lo = (long long)j * p.per, hi = lo + p.per;
            h[b].sub_begin = (int32_t)(lo < r.n ? lo : r.n);
            h[b].sub_end = (int32_t)(hi < r.n ? hi : r.n);
            h[b].comp_pad = p.mode == 1 ? 1 : 0;
            h[b].pad = 0;
            if (p.mode == 0) {
                h[b].comp_out = nullptr;
            } else if (p.mode == 1) {
                h[b].comp_out = comp + (size_t)j * (size_t)r.k;
            } else {
                const int len = h[b].sub_end - h[b].sub_begin;
                h[b].comp_out = comp;
                list_ptr[j] = comp;
                list_len[j] = len < r.k ? len : r.k;
                comp += (size_t)list_len[j];
            }
        }
        if (p.mode == 1) {
            hm[m].comp_in = first;
            hm[m].score = r.score;
            hm[m].out_idx = r.out_idx;
            hm[m].out_score = r.out_score;
            hm[m].n_comp = p.s * r.k;
            hm[m].n = r.n;
            hm[m].k = r.k;
            hm[m].pad = 0;
            comp += (size_t)p.s * (size_t)r.k;
            ++m;
        } else if (p.mode == 2) {
            int lists = p.s, lv = 0;
            while (lists > 1) {
                const int pairs = lists / 2;
                for (int q = 0; q < pairs; ++q) {
                    TopkPairDesc &t = hp[level_fill[lv]++];
                    t.a = list_ptr[2 * q];
                    t.b = list_ptr[2 * q + 1];
                    t.la = list_len[2 * q];
                    t.lb = list_len[2 * q + 1];
                    const long long both = (long long)t.la + t.lb;
                    if (both > level_entries[lv])
                        level_entries[lv] = (int)both;
                    t.lo = (int32_t)(both < r.k ? both : r.k);
                    t.k = r.k;
                    t.score = r.score;
                    t.out_idx = r.out_idx;
                    t.out_score = r.out_score;
                    if (lists == 2) {
                        t.out = nullptr;                      // last level: the answer itself
                    } else {
                        t.out = comp;
                        comp += (size_t)r.k;
                    }
                    list_ptr[q] = t.out;
                    list_len[q] = t.lo;
                }
                if (lists & 1) {                              // odd one out moves up as it is
                    list_ptr[pairs] = list_ptr[lists - 1];
                    list_len[pairs] = list_len[lists - 1];
                }
                lists = pairs + (lists & 1);
                ++lv;
            }
        }
    }
    if ((size_t)(comp - (unsigned long long *)ctx->scratch[kScratchTopk]) > comp_total || b != n_blocks || m != n_merge)
        return fail(FS_EDEVICE, "fs_topk: internal plan mismatch");
    rc = commit_desc(db, total_bytes, stream);
    if (rc != FS_OK)
        return rc;
    prof_start(kKernTopk, stream);
    rc = launch_topk((const TopkDesc *)db.dev, (int)n_blocks, max_k, stream);
    if (rc == FS_OK && n_merge)
        rc = launch_topk_merge((const TopkMergeDesc *)((const char *)db.dev + merge_off),
                               (int)n_merge, max_comp, stream);
    for (int lv = 0; lv < n_levels && rc == FS_OK; ++lv)
        rc = launch_topk_pairs((const TopkPairDesc *)((const char *)db.dev + path_off) + level_at[lv],
                               (int)level_pairs[lv], level_entries[lv], stream);
    prof_stop(stream);
    const int rc2 = finish_desc(db, stream);
    return rc != FS_OK ? rc : rc2;
}

// ---- layout helper -----------------------------------------------------------------------------
extern "C" int fs_pack_colblock64(const float *rowmajor, int64_t n_rows, int32_t n_features,
                                  float *out, void *stream)
{
    if (n_rows < 0 || n_rows >= ((int64_t)1 << 31))
        return fail(FS_EINVAL, "fs_pack_colblock64: n_rows %lld outside [0, 2^31)", (long long)n_rows);
    if (n_features < 1 || n_features > FS_MAX_FEATURES)
        return fail(FS_EINVAL, "fs_pack_colblock64: n_features %d outside [1, %d]", n_features,
                    FS_MAX_FEATURES);
    if (n_rows == 0)
        return FS_OK;
    if (!rowmajor || !out)
        return fail(FS_EINVAL, "fs_pack_colblock64: NULL buffer");
    prof_start(kKernPack, (hipStream_t)stream);
    int rc = launch_pack_colblock64(rowmajor, n_rows, n_features, out, (hipStream_t)stream);
    prof_stop((hipStream_t)stream);
    return rc;
}
