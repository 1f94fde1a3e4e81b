// C ABI of libmf_sgd (declared in include/mf_sgd.h): argument checks, state machine
// (created -> initialised -> loaded), workspace layout and the stratum scheduler that turns one
// epoch of Algorithm 1's training phase into one kernel launch per stratum.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/mf_sgd.h"
#include "mf_internal.h"

// The Hogwild LDS kernels keep only the touched columns of a strip in LDS when at most this
// share of all strip columns is touched (or when whole strips do not fit).
constexpr double kSparseStripShare = 0.75;
// The same for the deterministic LDS kernels, which move a packed strip column by column
// (measured: 10 % slower than whole strips with 61 % of the columns touched, 2 % faster with 18 %).
constexpr double kDetSparseStripShare = 0.3;

struct mf_ctx {
    int device = 0;
    int compute_units = 256;
    hipStream_t stream = nullptr;
    std::string err;

    // factors (caller-owned device buffers)
    bool inited = false;
    int64_t m = 0, n = 0;
    int32_t k = 0, dtype = MF_F32;
    void* dP = nullptr;
    void* dQt = nullptr;

    double touched_share = 1.0;   // touched columns / strip columns over the blocks of the last load
    int32_t max_slots = 0;        // most touched columns of any block (when the table was made)
    uint32_t* touched = nullptr;  // the table of touched columns of the last load (null: not made)
    int32_t touched_words = 0;
    // partition and schedules
    bool loaded = false;
    mf::Partition part;
    mf::Schedule sched[2];   // indexed by MF_MODE_*
    mf::LdsSchedule lds;     // Hogwild with the Qt strip in LDS
    mf::LdsSchedule det_lds; // deterministic mode with the Qt strip in LDS
    int32_t* dU = nullptr;
    int32_t* dV = nullptr;
    float* dR = nullptr;

    // options
    int32_t hogwild_chunk = 0;   // 0 = at most lds_waves chunks per block
    int32_t xcd_affinity = 1;
    int32_t profile = 0;
    int32_t hogwild_kernel = MF_HOGWILD_AUTO;
    int32_t det_kernel = MF_KERNEL_AUTO;
    int32_t use_ring = 1;                 // one launch per epoch when the grid allows it
    int64_t spin_limit = (int64_t)1 << 22;
    int32_t ring_resident[2] = {-1, -1};  // workgroups of the ring kernel the device holds at once, per mode
    int32_t ring_epochs = 0;              // epochs run by the ring kernel since mf_load_blocks
    bool ring_gave_up = false;            // a bounded wait expired on this load: per-stratum launches from now on
    bool epochs_since_check = false;      // SGD kernels were enqueued since the device flags were last read
    uint32_t* d_perm = nullptr;           // packed -> original position when the partition was made on the device
    int32_t* d_order = nullptr;           // 2 * grid_c numbers inside the workspace: order, inverse
    int32_t* d_ring_done = nullptr;       // grid_r counters + the abort flag + the range flag, inside the workspace
    int32_t lds_chunk = 0;   // 0 = one chunk per wavefront
    int32_t lds_waves = 16;    // option value (upper bound of the workspace estimates)
    bool lds_waves_set = false;  // the caller chose it
    int32_t lds_waves_used = 16; // what the loaded LDS work list was built for
    int32_t lds_prefetch = 0;  // 0 = by the size of P, else 4 or 8
    int32_t pack_strips = 1;   // MF_OPT_PACK_STRIPS: 0 never, 1 where it pays, 2 wherever possible
    uint64_t row_seed = 0;     // 0 = rows of a block in ascending order

    // library-owned device buffer: RMSE partials followed by the final sum
    double* d_partials = nullptr;

    // streamed mode (mf_load_blocks_streamed): the packed ratings stay in pinned host memory and
    // travel stratum by stratum into two device buffers while the stratum before is computed
    bool streamed = false;
    char* h_packed = nullptr;             // pinned, library-owned: stratum after stratum, each as its row
                                          // indices, then its column indices, then its values
    char* d_stream_buf[2] = {nullptr, nullptr};   // library-owned, 12 bytes x the largest stratum each
    int64_t stratum_cap = 0;                      // ratings one buffer holds
    int32_t stream_group = 1;                     // strata per transfer
    hipStream_t copy_stream = nullptr;            // default priority
    hipEvent_t copied[2] = {nullptr, nullptr}, consumed[2] = {nullptr, nullptr};
    bool consumed_recorded[2] = {false, false};

    // profiling events (start, stop) of the launches since the last mf_profile_read
    std::vector<std::pair<hipEvent_t, hipEvent_t>> events;
    size_t events_used = 0;
};

// Scratch of mf_rmse_noalloc: one partial sum per wavefront of the RMSE kernel's fixed launch shape.
// Every GPU the library runs on holds its own copy (64 KiB) at its own address until the process
// ends; the array's name is only a host-side handle, kernels and copies take the address that
// hipGetSymbolAddress returned with that GPU current (kept in g_scratch_addr, resolved in mf_create).
static __device__ __align__(256) double scratch[mf::kRmsePartials];
constexpr int kMaxDevices = 64;
static double* g_scratch_addr[kMaxDevices] = {};

namespace {

int fail(mf_ctx* ctx, int code, const std::string& msg)
{
    if (ctx) ctx->err = msg;
    return code;
}

int fail_hip(mf_ctx* ctx, const char* what, hipError_t e)
{
    return fail(ctx, MF_EDEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

#define MF_HIP(ctx, call)                                      \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return fail_hip(ctx, #call, e_); \
    } while (0)

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

void release_streaming(mf_ctx* ctx)
{
    if (ctx->copy_stream) (void)hipStreamSynchronize(ctx->copy_stream);
    for (int i = 0; i < 2; ++i) {
        if (ctx->d_stream_buf[i]) (void)hipFree(ctx->d_stream_buf[i]);
        ctx->d_stream_buf[i] = nullptr;
        ctx->consumed_recorded[i] = false;
    }
    if (ctx->h_packed) (void)hipHostFree(ctx->h_packed);
    ctx->h_packed = nullptr;
    ctx->streamed = false;
}

bool valid_k(int32_t k) { return k == 32 || k == 64 || k == 128 || k == 256; }

struct Layout {
    size_t off_u, off_v, off_r, off_perm, off_begin[2], off_len[2], off_lds_begin, off_lds_len, off_lds_blocks,
        off_dlds_begin, off_dlds_len, off_dlds_blocks, off_ring[2], off_ring_done, off_order, off_hot, off_touched, total;
    int64_t cap[2], lds_cap, lds_blocks_cap, hot_cap;
    int32_t touched_words;
};

// Bit words per block of the table of touched columns: room for the widest strip the one-launch
// Hogwild kernel can pack (64 pieces of 64 words per wavefront, 16 wavefronts) with this k and
// storage type (before mf_init: the most the table can have).  0 in streamed mode, where the
// table is not built.
int32_t touched_words_bound(const mf_ctx* ctx)
{
    if (!ctx->inited) return mf::kMaxTouchedWords;
    const int64_t words_per_column = (int64_t)ctx->k * (ctx->dtype == MF_F16 ? 2 : 4) / 4;
    const int64_t cols = std::min<int64_t>(ctx->n, (int64_t)64 * 64 * 16 / words_per_column);
    return (int32_t)std::min<int64_t>(mf::kMaxTouchedWords, (cols + 31) / 32);
}

Layout make_layout(const mf_ctx* ctx, int64_t nnz, int32_t gr, int32_t gc, bool resident = true)
{
    const int32_t chunk = ctx->hogwild_chunk, lds_chunk = ctx->lds_chunk, lds_waves = ctx->lds_waves;
    const size_t packed = resident ? (size_t)nnz * 4 : 0;   // streamed mode keeps the ratings on the host
    Layout l;
    l.cap[MF_MODE_DET] = mf::det_entries_bound(gr, gc);
    l.cap[MF_MODE_HOGWILD] = mf::hogwild_entries_bound(nnz, gr, gc, chunk, lds_waves);
    l.lds_cap = mf::lds_entries_bound(nnz, gr, gc, lds_chunk, lds_waves);
    l.lds_blocks_cap = (int64_t)gr * gc;
    l.hot_cap = mf::lds_hot_bound(nnz, gr, gc);
    size_t off = 0;
    l.off_u = off; off += align_up(packed);
    l.off_v = off; off += align_up(packed);
    l.off_r = off; off += align_up(packed);
    l.off_perm = off; off += align_up(packed);   // written by mf_load_blocks_device only
    for (int mode = 0; mode < 2; ++mode) {
        l.off_begin[mode] = off; off += align_up((size_t)l.cap[mode] * 8);
        l.off_len[mode] = off; off += align_up((size_t)l.cap[mode] * 4);
    }
    l.off_lds_begin = off; off += align_up((size_t)l.lds_cap * 8);
    l.off_lds_len = off; off += align_up((size_t)l.lds_cap * 4);
    l.off_lds_blocks = off; off += align_up((size_t)l.lds_blocks_cap * sizeof(mf::LdsBlock));
    l.off_dlds_begin = off; off += align_up((size_t)l.lds_blocks_cap * 8);   // one entry per block
    l.off_dlds_len = off; off += align_up((size_t)l.lds_blocks_cap * 4);
    l.off_dlds_blocks = off; off += align_up((size_t)l.lds_blocks_cap * sizeof(mf::LdsBlock));
    for (int which = 0; which < 2; ++which) {
        l.off_ring[which] = off; off += align_up((size_t)l.lds_blocks_cap * sizeof(mf::LdsBlock));
    }
    l.off_ring_done = off; off += align_up(((size_t)gr + 2) * 4);
    l.off_order = off; off += align_up((size_t)gc * 2 * 4);   // stratum order of an epoch and its inverse
    l.off_hot = off; off += align_up((size_t)l.hot_cap * 8);   // cut rows of the Hogwild LDS work list
    l.touched_words = resident ? touched_words_bound(ctx) : 0;
    l.off_touched = off; off += align_up((size_t)l.lds_blocks_cap * l.touched_words * 4) + 256;   // + two counters
    l.total = off;
    return l;
}

// MF_OPT_PROFILE: an event before a launch (begin_launch_timing) and one after it (its return
// value, to be recorded by the caller); the pairs are read by mf_profile_read.
hipError_t begin_launch_timing(mf_ctx* ctx, hipEvent_t* after)
{
    *after = nullptr;
    if (!ctx->profile) return hipSuccess;
    if (ctx->events_used == ctx->events.size()) {
        hipEvent_t ev0 = nullptr, ev1 = nullptr;
        hipError_t e = hipEventCreate(&ev0);
        if (e == hipSuccess) e = hipEventCreate(&ev1);
        if (e != hipSuccess) return e;
        ctx->events.push_back({ev0, ev1});
    }
    *after = ctx->events[ctx->events_used].second;
    const hipEvent_t before = ctx->events[ctx->events_used].first;
    ctx->events_used += 1;
    return hipEventRecord(before, ctx->stream);
}

// After a synchronisation: read the two device flags the SGD kernels may raise.
//   abort flag: a workgroup of the one-launch-per-epoch kernel gave up waiting for its neighbour
//               (the device was shared, or the wait limit was set too low); the epoch was abandoned
//               half-applied.  The context falls back to one launch per stratum for this load.
//   range flag: the fixed-point strip of the Hogwild LDS kernel met a value of Qt (or of a row of P
//               kept beside it) of magnitude >= 64, or a single change of magnitude >= 4: the
//               training has diverged and values may have wrapped round.
// Both are cleared once reported.
int check_device_flags(mf_ctx* ctx)
{
    if (!ctx->loaded || !ctx->d_ring_done || !ctx->epochs_since_check) return MF_OK;
    int32_t flags[2] = {0, 0};
    hipError_t e = hipMemcpy(flags, ctx->d_ring_done + ctx->part.gr, 8, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(ctx, "reading the kernels' status flags", e);
    ctx->epochs_since_check = false;
    if (flags[0] == 0 && flags[1] == 0) return MF_OK;
    e = hipMemset(ctx->d_ring_done, 0, ((size_t)ctx->part.gr + 2) * 4);
    if (e != hipSuccess) return fail_hip(ctx, "clearing the kernels' status flags", e);
    ctx->ring_epochs = 0;
    if (flags[0] != 0) {
        ctx->ring_gave_up = true;
        return fail(ctx, MF_EDEVICE, "a workgroup of the one-launch-per-epoch kernel exceeded its wait limit (is the "
                                     "device shared?); that epoch was abandoned and the factors are in an undefined "
                                     "state; later epochs on this load use one launch per stratum");
    }
    return fail(ctx, MF_ERANGE, "the Hogwild LDS kernel met a value of magnitude >= 64 or a single change >= 4 in its "
                                "fixed-point strip: the training has diverged (lower lr or the initial scale)");
}

int check_grid(mf_ctx* ctx, int64_t nnz, int32_t gr, int32_t gc)
{
    if (nnz < 0 || nnz >= ((int64_t)1 << 31)) return fail(ctx, MF_EINVAL, "nnz must be in [0, 2^31)");
    if (gr < 1 || gc < 1 || gr > gc) return fail(ctx, MF_EINVAL, "need 1 <= grid_r <= grid_c");
    if ((int64_t)gr * gc >= ((int64_t)1 << 30)) return fail(ctx, MF_EINVAL, "grid too large");
    return MF_OK;
}

}  // namespace

extern "C" {

int mf_create(mf_ctx** out, int device, void* hip_stream)
{
    if (!out) return MF_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return MF_EDEVICE;
    mf_ctx* ctx = new (std::nothrow) mf_ctx();
    if (!ctx) return MF_ENOMEM;
    ctx->device = device;
    ctx->stream = (hipStream_t)hip_stream;
    if (hipSetDevice(device) != hipSuccess ||
        hipMalloc((void**)&ctx->d_partials, (mf::kRmsePartials + 1) * sizeof(double)) != hipSuccess) {
        delete ctx;
        return MF_EDEVICE;
    }
    if (device < kMaxDevices && !g_scratch_addr[device]) {
        // with this device current: where its copy of the static scratch array lives
        double* addr = nullptr;
        if (hipGetSymbolAddress((void**)&addr, HIP_SYMBOL(scratch)) != hipSuccess || !addr) {
            (void)hipFree(ctx->d_partials);
            delete ctx;
            return MF_EDEVICE;
        }
        g_scratch_addr[device] = addr;
    }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0)
        ctx->compute_units = cus;
    *out = ctx;
    return MF_OK;
}

int mf_destroy(mf_ctx* ctx)
{
    if (!ctx) return MF_EINVAL;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    for (auto& ev : ctx->events) {
        (void)hipEventDestroy(ev.first);
        (void)hipEventDestroy(ev.second);
    }
    if (ctx->d_partials) (void)hipFree(ctx->d_partials);
    release_streaming(ctx);
    for (int i = 0; i < 2; ++i) {
        if (ctx->copied[i]) (void)hipEventDestroy(ctx->copied[i]);
        if (ctx->consumed[i]) (void)hipEventDestroy(ctx->consumed[i]);
    }
    if (ctx->copy_stream) (void)hipStreamDestroy(ctx->copy_stream);
    delete ctx;
    return MF_OK;
}

const char* mf_last_error(const mf_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int mf_set_option(mf_ctx* ctx, int32_t option, int64_t value)
{
    if (!ctx) return MF_EINVAL;
    switch (option) {
        case MF_OPT_HOGWILD_CHUNK:
            if (value < 0 || value > (1 << 20)) return fail(ctx, MF_EINVAL, "chunk must be in [0, 2^20]");
            ctx->hogwild_chunk = (int32_t)value;
            return MF_OK;
        case MF_OPT_XCD_AFFINITY:
            ctx->xcd_affinity = value ? 1 : 0;
            return MF_OK;
        case MF_OPT_PROFILE:
            ctx->profile = value ? 1 : 0;
            return MF_OK;
        case MF_OPT_HOGWILD_KERNEL:
            if (value < MF_HOGWILD_AUTO || value > MF_HOGWILD_LDS) return fail(ctx, MF_EINVAL, "unknown Hogwild kernel");
            ctx->hogwild_kernel = (int32_t)value;
            return MF_OK;
        case MF_OPT_DET_KERNEL:
            if (value < MF_KERNEL_AUTO || value > MF_KERNEL_LDS) return fail(ctx, MF_EINVAL, "unknown kernel choice");
            ctx->det_kernel = (int32_t)value;
            return MF_OK;
        case MF_OPT_RING:
            ctx->use_ring = value ? 1 : 0;
            return MF_OK;
        case MF_OPT_RING_SPIN_LIMIT:
            if (value < 1) return fail(ctx, MF_EINVAL, "spin limit must be positive");
            ctx->spin_limit = value;
            return MF_OK;
        case MF_OPT_LDS_CHUNK:
            if (value < 0 || value > (1 << 20)) return fail(ctx, MF_EINVAL, "chunk must be in [0, 2^20]");
            ctx->lds_chunk = (int32_t)value;
            return MF_OK;
        case MF_OPT_LDS_WAVES:
            if (value < 1 || value > 16) return fail(ctx, MF_EINVAL, "wavefronts per workgroup must be in [1, 16]");
            ctx->lds_waves = (int32_t)value;
            ctx->lds_waves_set = true;
            return MF_OK;
        case MF_OPT_ROW_ORDER_SEED:
            if (value < 0) return fail(ctx, MF_EINVAL, "the seed must not be negative");
            ctx->row_seed = (uint64_t)value;
            return MF_OK;
        case MF_OPT_LDS_PREFETCH:
            if (value != 0 && value != 4 && value != 8) return fail(ctx, MF_EINVAL, "MF_OPT_LDS_PREFETCH is 0, 4 or 8");
            ctx->lds_prefetch = (int32_t)value;
            return MF_OK;
        case MF_OPT_PACK_STRIPS:
            if (value < 0 || value > 2) return fail(ctx, MF_EINVAL, "MF_OPT_PACK_STRIPS is 0, 1 or 2");
            ctx->pack_strips = (int32_t)value;
            return MF_OK;
    }
    return fail(ctx, MF_EINVAL, "unknown option");
}

int mf_init(mf_ctx* ctx, int64_t m, int64_t n, int32_t k, int32_t dtype, void* dP, void* dQt,
            uint64_t seed, float scale)
{
    if (!ctx) return MF_EINVAL;
    if (m < 1 || n < 1 || m >= ((int64_t)1 << 31) || n >= ((int64_t)1 << 31))
        return fail(ctx, MF_EINVAL, "m and n must be in [1, 2^31)");
    if (!valid_k(k)) return fail(ctx, MF_EINVAL, "k must be 32, 64, 128 or 256");
    if (dtype != MF_F32 && dtype != MF_F16) return fail(ctx, MF_EINVAL, "dtype must be MF_F32 or MF_F16");
    if (!dP || !dQt) return fail(ctx, MF_EINVAL, "null factor buffer");
    if (((uintptr_t)dP | (uintptr_t)dQt) & 15) return fail(ctx, MF_EINVAL, "factor buffers must be 16-byte aligned");
    if (!(scale == scale)) return fail(ctx, MF_EINVAL, "scale is NaN");
    MF_HIP(ctx, hipSetDevice(ctx->device));
    ctx->inited = false;
    ctx->loaded = false;   // a partition belongs to the matrix shape it was made for
    if (scale >= 0.f) {
        MF_HIP(ctx, mf::launch_init(dtype, dP, m * k, seed, 0, scale, ctx->stream));
        MF_HIP(ctx, mf::launch_init(dtype, dQt, n * k, seed, 1, scale, ctx->stream));
    }
    ctx->m = m;
    ctx->n = n;
    ctx->k = k;
    ctx->dtype = dtype;
    ctx->dP = dP;
    ctx->dQt = dQt;
    ctx->inited = true;
    return MF_OK;
}

int mf_load_blocks_workspace(const mf_ctx* ctx, int64_t nnz, int32_t grid_r, int32_t grid_c,
                             size_t* bytes_out)
{
    if (!ctx || !bytes_out) return MF_EINVAL;
    int rc = check_grid(const_cast<mf_ctx*>(ctx), nnz, grid_r, grid_c);
    if (rc) return rc;
    *bytes_out = make_layout(ctx, nnz, grid_r, grid_c).total;
    return MF_OK;
}

namespace {

int check_load(mf_ctx* ctx, const void* rows, const void* cols, const void* vals, int64_t nnz, int32_t grid_r,
               int32_t grid_c, int32_t split, void* d_workspace, size_t workspace_bytes, Layout& lay,
               bool resident = true)
{
    if (!ctx->inited) return fail(ctx, MF_ESTATE, "mf_load_blocks before mf_init");
    int rc = check_grid(ctx, nnz, grid_r, grid_c);
    if (rc) return rc;
    if (grid_r > ctx->m || grid_c > ctx->n) return fail(ctx, MF_EINVAL, "grid exceeds the matrix size");
    if (split < MF_SPLIT_EQUAL_WIDTH || split > MF_SPLIT_NNZ_WIDTH_BALANCED) return fail(ctx, MF_EINVAL, "unknown split rule");
    if (nnz > 0 && (!rows || !cols || !vals)) return fail(ctx, MF_EINVAL, "null rating array");
    if (!d_workspace) return fail(ctx, MF_EINVAL, "null workspace");
    if ((uintptr_t)d_workspace & 255) return fail(ctx, MF_EINVAL, "workspace must be 256-byte aligned");
    lay = make_layout(ctx, nnz, grid_r, grid_c, resident);
    if (workspace_bytes < lay.total) return fail(ctx, MF_ENOMEM, "workspace too small");
    return MF_OK;
}

// The partition and the packed arrays exist (ctx->part; `rs` = where the row runs begin):
// derive the work lists and put them into the workspace.
// Which columns of its strip every block touches (resident ratings only): the table the
// Hogwild LDS kernels pack their strips with, made before the work lists because the room
// the packed strips leave in LDS decides how many rows a block may cut.  Sets ctx->lds.d_touched
// when packing is possible and pays.
int make_touched_table(mf_ctx* ctx, const Layout& lay, char* base)
{
    ctx->lds.d_touched = nullptr;
    ctx->lds.touched_words = 0;
    ctx->det_lds.d_touched = nullptr;
    ctx->det_lds.touched_words = 0;
    ctx->touched_share = 1.0;
    ctx->max_slots = 0;
    ctx->touched = nullptr;
    ctx->touched_words = 0;
    const mf::Partition& part = ctx->part;
    const int32_t widest = mf::widest_strip(part);
    const int32_t words = (widest + 31) / 32;
    if (!ctx->pack_strips || ctx->streamed || !ctx->dV || part.nnz == 0 || words < 1 || words > lay.touched_words)
        return MF_OK;
    // Hogwild form: a wavefront's 64 consecutive words of a strip have to lie in one column, and
    // its 64 piece bits have to cover the widest strip (the deterministic form moves a strip
    // column by column and has no such limits)
    const int64_t words_per_column = (int64_t)ctx->k * (ctx->dtype == MF_F16 ? 2 : 4) / 4;
    const bool shape_ok = words_per_column % 64 == 0 &&
                          (int64_t)widest * words_per_column <= (int64_t)64 * 64 * ctx->lds_waves_used;
    std::vector<mf::LdsBlock> ranges;
    for (int32_t st = 0; st < part.gc; ++st)
        for (int32_t a = 0; a < part.gr; ++a) {
            const int64_t L = (int64_t)st * part.gr + a;
            const int64_t size = part.block_ptr[(size_t)L + 1] - part.block_ptr[(size_t)L];
            if (size == 0) continue;
            const int32_t b = (a + st) % part.gc;
            ranges.push_back(mf::LdsBlock{part.block_ptr[(size_t)L], (int32_t)size, part.col_bounds[(size_t)b],
                                          part.col_bounds[(size_t)b + 1] - part.col_bounds[(size_t)b], 0, (int32_t)L, 0});
        }
    // the list travels through the place of the work list's block descriptors, which are written later
    mf::LdsBlock* d_ranges = (mf::LdsBlock*)(base + lay.off_lds_blocks);
    uint32_t* table = (uint32_t*)(base + lay.off_touched);
    unsigned long long* totals =
        (unsigned long long*)(base + lay.off_touched + align_up((size_t)lay.lds_blocks_cap * lay.touched_words * 4));
    MF_HIP(ctx, hipMemcpy(d_ranges, ranges.data(), ranges.size() * sizeof(mf::LdsBlock), hipMemcpyHostToDevice));
    MF_HIP(ctx, mf::launch_fill_i32((int32_t*)table, (int64_t)lay.lds_blocks_cap * words, 0, ctx->stream));
    MF_HIP(ctx, mf::launch_fill_i32((int32_t*)totals, 8, 0, ctx->stream));
    MF_HIP(ctx, mf::launch_mark_touched(d_ranges, (int64_t)ranges.size(), ctx->dV, table, words, totals, ctx->stream));
    MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    unsigned long long sums[3] = {0, 0, 0};
    MF_HIP(ctx, hipMemcpy(sums, totals, sizeof(sums), hipMemcpyDeviceToHost));
    if (sums[1] > 0) ctx->touched_share = (double)sums[0] / (double)sums[1];
    ctx->touched = table;
    ctx->touched_words = words;
    ctx->max_slots = (int32_t)sums[2];
    // Packing costs a little on every step (the map of a strip, a table look-up per 64 ratings),
    // which pays when a good part of the columns can be left out (measured: a gain of 8-10 % with
    // 45 % of the columns touched, a loss of 7 % with nearly all touched) -- and is the only way
    // when the whole strip does not fit.
    const size_t dense = mf::lds_strip_bytes(ctx->k, widest);
    const size_t packed = mf::lds_strip_bytes(ctx->k, (int32_t)sums[2]) + (size_t)words * 64;
    if (shape_ok && packed <= mf::kLdsBudget && (ctx->pack_strips == 2 || ctx->touched_share <= kSparseStripShare || dense > mf::kLdsBudget)) {
        ctx->lds.d_touched = table;
        ctx->lds.touched_words = words;
    }
    return MF_OK;
}

int finish_load(mf_ctx* ctx, const Layout& lay, char* base, const mf::RowStarts& rs)
{
    ctx->lds_waves_used = ctx->lds_waves;
    if (!ctx->lds_waves_set && ctx->lds_chunk == 0 && ctx->part.nnz > 0) {
        // eight ratings per wavefront and block at least (measured on the MovieLens-shaped
        // configuration: 16 wavefronts are best for blocks of 197 and of 151 ratings)
        int64_t blocks = 0;
        for (size_t L = 0; L + 1 < ctx->part.block_ptr.size(); ++L)
            blocks += ctx->part.block_ptr[L + 1] > ctx->part.block_ptr[L];
        const int64_t per_block = ctx->part.nnz / std::max<int64_t>(1, blocks);
        ctx->lds_waves_used = (int32_t)std::min<int64_t>(ctx->lds_waves, std::max<int64_t>(4, (per_block + 4) / 8));
    }
    int rc = make_touched_table(ctx, lay, base);
    if (rc) return rc;
    try {
        mf::build_det_schedule(ctx->part, ctx->xcd_affinity != 0, ctx->sched[MF_MODE_DET]);
        mf::build_hogwild_schedule(ctx->part, rs, ctx->hogwild_chunk, ctx->lds_waves, ctx->xcd_affinity != 0,
                                   ctx->sched[MF_MODE_HOGWILD]);
        // cut rows stay in LDS beside the strip, as many per block as the widest strip (packed: the
        // most touched columns of a block, and the column table) leaves room for
        const int64_t widest = ctx->lds.d_touched
                                   ? (int64_t)mf::lds_strip_bytes(ctx->k, ctx->max_slots) + (int64_t)ctx->lds.touched_words * 64
                                   : (int64_t)mf::lds_strip_bytes(ctx->k, mf::widest_strip(ctx->part));
        const int32_t hot_slots = (int32_t)std::max<int64_t>(
            0, std::min<int64_t>(mf::kMaxHotRows, ((int64_t)mf::kLdsBudget - widest) / ((int64_t)ctx->k * 4)));
        mf::build_lds_schedule(ctx->part, rs, ctx->lds_chunk, ctx->lds_waves_used, hot_slots, ctx->lds);
        mf::build_det_lds_schedule(ctx->part, ctx->det_lds);
    } catch (const std::bad_alloc&) {
        return fail(ctx, MF_ENOMEM, "host allocation failed while building the work lists");
    }
    for (int mode = 0; mode < 2; ++mode) {
        mf::Schedule& s = ctx->sched[mode];
        if ((int64_t)s.begin.size() > lay.cap[mode])
            return fail(ctx, MF_ENOMEM, "schedule larger than its workspace bound");
        s.d_begin = (int64_t*)(base + lay.off_begin[mode]);
        s.d_len = (int32_t*)(base + lay.off_len[mode]);
        if (!s.begin.empty()) {
            MF_HIP(ctx, hipMemcpy(s.d_begin, s.begin.data(), s.begin.size() * 8, hipMemcpyHostToDevice));
            MF_HIP(ctx, hipMemcpy(s.d_len, s.len.data(), s.len.size() * 4, hipMemcpyHostToDevice));
        }
    }
    for (int which = 0; which < 2; ++which) {
        mf::LdsSchedule& l = which ? ctx->det_lds : ctx->lds;
        const int64_t cap = which ? lay.lds_blocks_cap : lay.lds_cap;
        if ((int64_t)l.begin.size() > cap || (int64_t)l.blocks.size() > lay.lds_blocks_cap)
            return fail(ctx, MF_ENOMEM, "schedule larger than its workspace bound");
        l.d_begin = (int64_t*)(base + (which ? lay.off_dlds_begin : lay.off_lds_begin));
        l.d_len = (int32_t*)(base + (which ? lay.off_dlds_len : lay.off_lds_len));
        l.d_blocks = (mf::LdsBlock*)(base + (which ? lay.off_dlds_blocks : lay.off_lds_blocks));
        l.d_ring = (mf::LdsBlock*)(base + lay.off_ring[which]);
        l.d_hot = (int64_t*)(base + lay.off_hot);
        if ((int64_t)l.hot_pos.size() > lay.hot_cap) return fail(ctx, MF_ENOMEM, "schedule larger than its workspace bound");
        if (!which && !l.hot_pos.empty())
            MF_HIP(ctx, hipMemcpy(l.d_hot, l.hot_pos.data(), l.hot_pos.size() * 8, hipMemcpyHostToDevice));
        MF_HIP(ctx, hipMemcpy(l.d_ring, l.ring.data(), l.ring.size() * sizeof(mf::LdsBlock), hipMemcpyHostToDevice));
        if (!l.begin.empty()) {
            MF_HIP(ctx, hipMemcpy(l.d_begin, l.begin.data(), l.begin.size() * 8, hipMemcpyHostToDevice));
            MF_HIP(ctx, hipMemcpy(l.d_len, l.len.data(), l.len.size() * 4, hipMemcpyHostToDevice));
            MF_HIP(ctx, hipMemcpy(l.d_blocks, l.blocks.data(), l.blocks.size() * sizeof(mf::LdsBlock),
                                  hipMemcpyHostToDevice));
        }
    }
    ctx->d_ring_done = (int32_t*)(base + lay.off_ring_done);
    ctx->d_order = (int32_t*)(base + lay.off_order);
    MF_HIP(ctx, hipMemset(ctx->d_ring_done, 0, ((size_t)ctx->part.gr + 2) * 4));
    ctx->ring_epochs = 0;
    ctx->ring_gave_up = false;
    ctx->epochs_since_check = false;
    ctx->ring_resident[0] = ctx->ring_resident[1] = -1;
    ctx->loaded = true;
    return MF_OK;
}

}  // namespace

int mf_load_blocks(mf_ctx* ctx, const int32_t* rows, const int32_t* cols, const float* vals,
                   int64_t nnz, int32_t grid_r, int32_t grid_c, int32_t split, void* d_workspace,
                   size_t workspace_bytes)
{
    if (!ctx) return MF_EINVAL;
    Layout lay;
    int rc = check_load(ctx, rows, cols, vals, nnz, grid_r, grid_c, split, d_workspace, workspace_bytes, lay);
    if (rc) return rc;
    MF_HIP(ctx, hipSetDevice(ctx->device));
    ctx->loaded = false;
    MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    release_streaming(ctx);

    std::vector<int32_t> pu, pv;
    std::vector<float> pr;
    try {
        std::string err;
        rc = mf::build_partition(rows, cols, vals, nnz, ctx->m, ctx->n, grid_r, grid_c, split, ctx->row_seed, ctx->part,
                                 pu, pv, pr, err);
        if (rc) return fail(ctx, rc, err);
    } catch (const std::bad_alloc&) {
        return fail(ctx, MF_ENOMEM, "host allocation failed while partitioning");
    }

    char* base = (char*)d_workspace;
    ctx->dU = (int32_t*)(base + lay.off_u);
    ctx->dV = (int32_t*)(base + lay.off_v);
    ctx->dR = (float*)(base + lay.off_r);
    // the stream may still be running an epoch that reads the old contents of the workspace
    MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (nnz > 0) {
        MF_HIP(ctx, hipMemcpy(ctx->dU, pu.data(), (size_t)nnz * 4, hipMemcpyHostToDevice));
        MF_HIP(ctx, hipMemcpy(ctx->dV, pv.data(), (size_t)nnz * 4, hipMemcpyHostToDevice));
        MF_HIP(ctx, hipMemcpy(ctx->dR, pr.data(), (size_t)nnz * 4, hipMemcpyHostToDevice));
    }
    ctx->d_perm = nullptr;
    mf::RowStarts rs;
    mf::row_starts_from_rows(pu.data(), nnz, rs);
    return finish_load(ctx, lay, base, rs);
}

int mf_load_blocks_device(mf_ctx* ctx, const int32_t* d_rows, const int32_t* d_cols, const float* d_vals,
                          int64_t nnz, int32_t grid_r, int32_t grid_c, int32_t split, void* d_workspace,
                          size_t workspace_bytes)
{
    if (!ctx) return MF_EINVAL;
    Layout lay;
    int rc = check_load(ctx, d_rows, d_cols, d_vals, nnz, grid_r, grid_c, split, d_workspace, workspace_bytes, lay);
    if (rc) return rc;
    MF_HIP(ctx, hipSetDevice(ctx->device));
    ctx->loaded = false;
    MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    release_streaming(ctx);
    char* base = (char*)d_workspace;
    ctx->dU = (int32_t*)(base + lay.off_u);
    ctx->dV = (int32_t*)(base + lay.off_v);
    ctx->dR = (float*)(base + lay.off_r);
    MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    mf::RowStarts rs;
    ctx->d_perm = (uint32_t*)(base + lay.off_perm);
    try {
        std::string err;
        rc = mf::build_partition_device(d_rows, d_cols, d_vals, nnz, ctx->m, ctx->n, grid_r, grid_c, split,
                                        ctx->row_seed, ctx->dU, ctx->dV, ctx->dR, ctx->d_perm, ctx->part, rs, ctx->stream, err);
        if (rc) return fail(ctx, rc, err);
    } catch (const std::bad_alloc&) {
        return fail(ctx, MF_ENOMEM, "host allocation failed while partitioning");
    }
    return finish_load(ctx, lay, base, rs);
}

int mf_load_blocks_streamed_workspace(const mf_ctx* ctx, int64_t nnz, int32_t grid_r, int32_t grid_c,
                                      size_t* bytes_out)
{
    if (!ctx || !bytes_out) return MF_EINVAL;
    int rc = check_grid(const_cast<mf_ctx*>(ctx), nnz, grid_r, grid_c);
    if (rc) return rc;
    *bytes_out = make_layout(ctx, nnz, grid_r, grid_c, false).total;
    return MF_OK;
}

int mf_load_blocks_streamed(mf_ctx* ctx, const int32_t* rows, const int32_t* cols, const float* vals,
                            int64_t nnz, int32_t grid_r, int32_t grid_c, int32_t split, void* d_workspace,
                            size_t workspace_bytes)
{
    if (!ctx) return MF_EINVAL;
    Layout lay;
    int rc = check_load(ctx, rows, cols, vals, nnz, grid_r, grid_c, split, d_workspace, workspace_bytes, lay, false);
    if (rc) return rc;
    MF_HIP(ctx, hipSetDevice(ctx->device));
    ctx->loaded = false;
    MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    release_streaming(ctx);

    std::vector<int32_t> pu, pv;
    std::vector<float> pr;
    try {
        std::string err;
        rc = mf::build_partition(rows, cols, vals, nnz, ctx->m, ctx->n, grid_r, grid_c, split, ctx->row_seed, ctx->part,
                                 pu, pv, pr, err);
        if (rc) return fail(ctx, rc, err);
    } catch (const std::bad_alloc&) {
        return fail(ctx, MF_ENOMEM, "host allocation failed while partitioning");
    }
    // the packed arrays go to pinned host memory; the device gets two buffers of the largest stratum
    int64_t largest = 1;
    for (int32_t st = 0; st < grid_c; ++st)
        largest = std::max(largest, ctx->part.block_ptr[(size_t)(st + 1) * grid_r] - ctx->part.block_ptr[(size_t)st * grid_r]);
    MF_HIP(ctx, hipHostMalloc((void**)&ctx->h_packed, std::max<size_t>((size_t)nnz * 12, 256), hipHostMallocDefault));
    for (int32_t st = 0; st < grid_c; ++st) {
        // one transfer per stratum: its three arrays lie one after the other
        const int64_t begin = ctx->part.block_ptr[(size_t)st * grid_r];
        const int64_t size = ctx->part.block_ptr[(size_t)(st + 1) * grid_r] - begin;
        char* dst = ctx->h_packed + (size_t)begin * 12;
        std::memcpy(dst, pu.data() + begin, (size_t)size * 4);
        std::memcpy(dst + (size_t)size * 4, pv.data() + begin, (size_t)size * 4);
        std::memcpy(dst + (size_t)size * 8, pr.data() + begin, (size_t)size * 4);
    }
    // strata per transfer: enough for about 4 MiB; a buffer holds that many of the largest stratum
    const int64_t average = std::max<int64_t>(1, nnz / grid_c);
    ctx->stream_group = (int32_t)std::max<int64_t>(1, std::min<int64_t>(grid_c, ((int64_t)(4 << 20) / 12 + average - 1) / average));
    ctx->stratum_cap = ((largest * ctx->stream_group) + 63) & ~(int64_t)63;
    for (int i = 0; i < 2; ++i) MF_HIP(ctx, hipMalloc((void**)&ctx->d_stream_buf[i], (size_t)ctx->stratum_cap * 12));
    if (!ctx->copy_stream) {
        MF_HIP(ctx, hipStreamCreateWithFlags(&ctx->copy_stream, hipStreamNonBlocking));
        for (int i = 0; i < 2; ++i) {
            MF_HIP(ctx, hipEventCreateWithFlags(&ctx->copied[i], hipEventDisableTiming));
            MF_HIP(ctx, hipEventCreateWithFlags(&ctx->consumed[i], hipEventDisableTiming));
        }
    }
    ctx->streamed = true;
    ctx->dU = ctx->dV = nullptr;
    ctx->dR = nullptr;
    ctx->d_perm = nullptr;
    mf::RowStarts rs;
    mf::row_starts_from_rows(pu.data(), nnz, rs);
    return finish_load(ctx, lay, (char*)d_workspace, rs);
}

int mf_get_partition(const mf_ctx* ctx, int64_t* perm, int64_t* block_ptr, int32_t* row_bounds,
                     int32_t* col_bounds)
{
    if (!ctx) return MF_EINVAL;
    if (!ctx->loaded) return fail(const_cast<mf_ctx*>(ctx), MF_ESTATE, "no partition loaded");
    const mf::Partition& p = ctx->part;
    if (perm && !p.perm.empty()) std::memcpy(perm, p.perm.data(), p.perm.size() * 8);
    if (perm && p.perm.empty() && ctx->d_perm && p.nnz > 0) {
        // partition made on the device: the permutation lives in the workspace as 32-bit numbers
        std::vector<uint32_t> narrow((size_t)p.nnz);
        hipError_t e = hipSetDevice(ctx->device);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e == hipSuccess) e = hipMemcpy(narrow.data(), ctx->d_perm, (size_t)p.nnz * 4, hipMemcpyDeviceToHost);
        if (e != hipSuccess) return fail_hip(const_cast<mf_ctx*>(ctx), "reading the permutation", e);
        for (int64_t i = 0; i < p.nnz; ++i) perm[i] = (int64_t)narrow[(size_t)i];
    }
    if (block_ptr) std::memcpy(block_ptr, p.block_ptr.data(), p.block_ptr.size() * 8);
    if (row_bounds) std::memcpy(row_bounds, p.row_bounds.data(), p.row_bounds.size() * 4);
    if (col_bounds) std::memcpy(col_bounds, p.col_bounds.data(), p.col_bounds.size() * 4);
    return MF_OK;
}

int mf_stratum_order(uint64_t seed, uint64_t epoch, int32_t grid_c, int32_t* order_out)
{
    if (grid_c < 1 || !order_out) return MF_EINVAL;
    auto mix = [](uint64_t z) { return mf::mix64(z); };
    const uint64_t base = mix(seed ^ (epoch * 0xD1B54A32D192ED03ULL));
    std::vector<std::pair<uint64_t, int32_t>> keyed((size_t)grid_c);
    for (int32_t s = 0; s < grid_c; ++s) keyed[(size_t)s] = {mix(base + (uint64_t)s), s};
    std::sort(keyed.begin(), keyed.end());
    for (int32_t t = 0; t < grid_c; ++t) order_out[t] = keyed[(size_t)t].second;
    return MF_OK;
}

namespace {

// What one epoch of `mode` launches for the loaded grid.
struct EpochPlan {
    bool hog = false;
    bool use_lds = false;          // the kernels that keep the block's strip of Qt in LDS
    bool ring = false;             // one launch per epoch
    bool short_prefetch = false;
    size_t lds_bytes = 0;
    int32_t waves = 1;             // wavefronts per workgroup
    int32_t kernel = 0;            // MF_KERNEL_ID_*
    int64_t launches = 0;          // per epoch
    bool packed = false;           // LDS kernels with only the touched columns of a strip in LDS
    int32_t slot_table_at = 0;     // packed: where the kernel's column table begins in LDS (32-bit words)
    const uint32_t* touched = nullptr;   // packed: the table of touched columns
    int32_t touched_words = 0;
    std::string note;
};

int plan_epoch(mf_ctx* ctx, int32_t mode, EpochPlan& p)
{
    // both modes take the kernel that keeps the block's strip of Qt in LDS whenever the widest
    // strip fits (the deterministic mode additionally wants several workgroups per compute unit
    // to be possible, since each of its workgroups is a single wavefront)
    p.hog = mode == MF_MODE_HOGWILD;
    // rows of P are requested 8 ratings ahead when they come from HBM, 4 when P is small enough to
    // be served from the L2s and the memory-side cache (fewer padded positions per batch)
    const size_t p_bytes = (size_t)ctx->m * ctx->k * (ctx->dtype == MF_F16 ? 2 : 4);
    p.short_prefetch = ctx->lds_prefetch == 4 || (ctx->lds_prefetch == 0 && p_bytes <= ((size_t)64 << 20));
    const mf::LdsSchedule& lsched = p.hog ? ctx->lds : ctx->det_lds;
    const size_t dense_bytes = mf::lds_strip_bytes(ctx->k, lsched.max_cols) + (size_t)lsched.max_hot * ctx->k * 4;
    const int32_t choice = p.hog ? ctx->hogwild_kernel : ctx->det_kernel;
    // the deterministic form runs one wavefront per workgroup: its strips may take the share of a
    // compute unit's LDS that lets all grid_r workgroups be resident -- 1, 2, 4, 8 or 16 per unit
    // (shares that divide the LDS evenly; allocations are rounded up to 2 KiB, and a one-launch
    // epoch whose workgroups do not all fit can only give up)
    int64_t per_unit = 1;
    while (per_unit < 16 && per_unit * ctx->compute_units < ctx->part.gr) per_unit *= 2;
    const size_t det_budget = (((size_t)160 * 1024 / (size_t)per_unit) & ~(size_t)2047) - 1024;
    const size_t budget = p.hog || choice == MF_KERNEL_LDS ? mf::kLdsBudget : std::min(mf::kLdsBudget, det_budget);
    const bool ring_allowed = ctx->use_ring && !ctx->ring_gave_up && ctx->part.nnz > 0 && !ctx->streamed;
    // packed strips, when the load made the table of touched columns: the Hogwild form as the load
    // decided (its work list was made for that room); the deterministic form when packing pays
    // or whole strips do not fit
    p.touched = p.hog ? lsched.d_touched : ctx->touched;
    p.touched_words = p.hog ? lsched.touched_words : ctx->touched_words;
    p.slot_table_at = (ctx->max_slots + lsched.max_hot) * ctx->k;
    const size_t packed_bytes = (size_t)p.slot_table_at * 4 + (size_t)p.touched_words * 64;
    p.packed = p.touched && choice != MF_KERNEL_GLOBAL && packed_bytes <= budget &&
               (p.hog || ctx->pack_strips == 2 || ctx->touched_share <= kDetSparseStripShare || dense_bytes > budget);
    p.lds_bytes = p.packed ? packed_bytes : dense_bytes;
    p.use_lds = choice != MF_KERNEL_GLOBAL && p.lds_bytes <= budget;
    if (!p.use_lds && choice == MF_KERNEL_LDS)
        return fail(ctx, MF_EINVAL, "the widest column strip of this grid does not fit the LDS");
    p.waves = p.use_lds ? (p.hog ? ctx->lds_waves_used : 1) : mf::kWavesPerGroup;
    std::string why;
    if (!p.use_lds && choice != MF_KERNEL_GLOBAL) {
        why = "the widest column strip (" + std::to_string(lsched.max_cols) + " columns, " + std::to_string(dense_bytes) +
              " bytes) exceeds the " + std::to_string(budget) + " bytes of LDS this mode uses per workgroup";
        if (p.touched)
            why += ", and so do the " + std::to_string(ctx->max_slots) + " columns (" + std::to_string(packed_bytes) +
                   " bytes) that the block with the most touched columns would keep";
        why += "; ";
    }
    if (p.use_lds && ring_allowed) {
        // one launch for the whole epoch if every block row's workgroup can be resident at once
        const int m_idx = p.hog ? 1 : 0;
        if (ctx->ring_resident[m_idx] < 0) {
            int resident = 0;
            MF_HIP(ctx, mf::launch_sgd_ring(ctx->dtype, ctx->k, !p.hog, p.short_prefetch, ctx->lds_waves_used, true, &resident,
                                            nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                            ctx->part.gr, ctx->part.gc, p.lds_bytes, 0.f, 0.f, nullptr, 0, nullptr, 0,
                                            nullptr, nullptr, nullptr, 0, 0, 1, ctx->stream));
            ctx->ring_resident[m_idx] = resident;
        }
        p.ring = ctx->part.gr <= ctx->ring_resident[m_idx];
        if (!p.ring)
            why += "the device holds " + std::to_string(ctx->ring_resident[m_idx]) + " workgroups of this shape at once, fewer than grid_r; ";

    } else if (p.use_lds && ctx->ring_gave_up) {
        why += "an earlier epoch of the one-launch kernel exceeded its wait limit; ";
    }
    if (p.ring) {
        p.kernel = MF_KERNEL_ID_RING_LDS;
        p.launches = 1;
    } else {
        p.kernel = p.use_lds ? MF_KERNEL_ID_BLOCK_LDS : MF_KERNEL_ID_CHUNKS;
        const std::vector<int64_t>& first = p.use_lds ? lsched.stratum_block : ctx->sched[mode].stratum_entry;
        p.launches = 0;
        for (int32_t st = 0; st < ctx->part.gc; ++st) p.launches += first[(size_t)st + 1] > first[(size_t)st];
    }
    static const char* const names[] = {"", "sgd_chunks", "sgd_block_lds", "sgd_ring_lds"};
    p.note = std::string(p.hog ? "MF_MODE_HOGWILD" : "MF_MODE_DET") + ": " + names[p.kernel] + ", " +
             std::to_string(p.launches) + " launch(es) per epoch, " + std::to_string(p.waves) +
             " wavefront(s) per workgroup" + (why.empty() ? "" : " (" + why.substr(0, why.size() - 2) + ")");
    if (p.packed && p.use_lds)
        p.note += "; keeps only the touched columns of a strip in LDS (" +
                  std::to_string((int)(ctx->touched_share * 100.0 + 0.5)) + " % of all strip columns)";
    if (!p.hog && p.kernel == MF_KERNEL_ID_CHUNKS && choice != MF_KERNEL_GLOBAL)
        p.note += "; this grid was not made for the deterministic mode: one wavefront per block and one launch per "
                  "stratum (mf_suggest_grid gives a grid whose strips fit)";
    return MF_OK;
}

}  // namespace

int mf_epoch_plan(mf_ctx* ctx, int32_t mode, int32_t* kernel_out, int64_t* launches_out, int32_t* waves_out)
{
    if (!ctx) return MF_EINVAL;
    if (!ctx->loaded) return fail(ctx, MF_ESTATE, "mf_epoch_plan before mf_load_blocks");
    if (mode != MF_MODE_DET && mode != MF_MODE_HOGWILD) return fail(ctx, MF_EINVAL, "unknown mode");
    MF_HIP(ctx, hipSetDevice(ctx->device));
    EpochPlan plan;
    int rc = plan_epoch(ctx, mode, plan);
    if (rc) return rc;
    if (kernel_out) *kernel_out = plan.kernel;
    if (launches_out) *launches_out = plan.launches;
    if (waves_out) *waves_out = plan.waves;
    ctx->err = plan.note;
    return MF_OK;
}

namespace {
int sgd_epochs(mf_ctx* ctx, float lr, float lambda, int32_t mode, const int32_t* stratum_order, int32_t n_epochs);
}

int mf_sgd_epoch(mf_ctx* ctx, float lr, float lambda, int32_t mode)
{
    return sgd_epochs(ctx, lr, lambda, mode, nullptr, 1);
}

int mf_sgd_epoch_ordered(mf_ctx* ctx, float lr, float lambda, int32_t mode, const int32_t* stratum_order)
{
    return sgd_epochs(ctx, lr, lambda, mode, stratum_order, 1);
}

int mf_sgd_epochs(mf_ctx* ctx, float lr, float lambda, int32_t mode, int32_t n_epochs)
{
    if (ctx && (n_epochs < 1 || n_epochs > 4096)) return fail(ctx, MF_EINVAL, "n_epochs must be in 1 .. 4096");
    return sgd_epochs(ctx, lr, lambda, mode, nullptr, n_epochs);
}

namespace {
int sgd_epochs(mf_ctx* ctx, float lr, float lambda, int32_t mode, const int32_t* stratum_order, int32_t n_epochs)
{
    if (!ctx) return MF_EINVAL;
    if (!ctx->loaded) return fail(ctx, MF_ESTATE, "mf_sgd_epoch before mf_load_blocks");
    if (mode != MF_MODE_DET && mode != MF_MODE_HOGWILD) return fail(ctx, MF_EINVAL, "unknown mode");
    if (!(lr == lr) || !(lambda == lambda)) return fail(ctx, MF_EINVAL, "lr or lambda is NaN");
    const int32_t gc = ctx->part.gc;
    std::vector<int32_t> inverse;
    if (stratum_order) {
        inverse.assign((size_t)gc, -1);
        for (int32_t t = 0; t < gc; ++t) {
            const int32_t st = stratum_order[t];
            if (st < 0 || st >= gc || inverse[(size_t)st] >= 0)
                return fail(ctx, MF_EINVAL, "stratum_order is not a permutation of 0 .. grid_c-1");
            inverse[(size_t)st] = t;
        }
    }
    MF_HIP(ctx, hipSetDevice(ctx->device));
    EpochPlan plan;
    int rc = plan_epoch(ctx, mode, plan);
    if (rc) return rc;
    const mf::Schedule& s = ctx->sched[mode];
    const bool hog = plan.hog, use_lds = plan.use_lds, short_prefetch = plan.short_prefetch;
    const size_t lds_bytes = plan.lds_bytes;
    const mf::LdsSchedule& lsched = hog ? ctx->lds : ctx->det_lds;
    int32_t* const d_flags = ctx->d_ring_done + ctx->part.gr;   // abort flag, range flag
    ctx->epochs_since_check = true;
    if (!plan.ring && n_epochs > 1) {
        // only the one-launch kernel runs epochs on end: here, one after the other
        for (int32_t e = 0; e < n_epochs; ++e) {
            rc = sgd_epochs(ctx, lr, lambda, mode, nullptr, 1);
            if (rc) return rc;
        }
        return MF_OK;
    }
    if (plan.ring) {
        if ((int64_t)n_epochs * ctx->part.gc > ((int64_t)1 << 29))
            return fail(ctx, MF_EINVAL, "n_epochs * grid_c exceeds the range of the step counters");
        if ((int64_t)(ctx->ring_epochs + n_epochs) * ctx->part.gc > ((int64_t)1 << 30)) {
            // the strata counters are about to run out of range: start them again from zero (a
            // kernel, not a memset node, so that the call may be captured into a graph)
            MF_HIP(ctx, mf::launch_fill_i32(ctx->d_ring_done, ctx->part.gr, 0, ctx->stream));
            ctx->ring_epochs = 0;
        }
        if (stratum_order) {
            // the order and its inverse go to the workspace; an epoch that may still be reading
            // the previous order has to finish first
            MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
            MF_HIP(ctx, hipMemcpy(ctx->d_order, stratum_order, (size_t)gc * 4, hipMemcpyHostToDevice));
            MF_HIP(ctx, hipMemcpy(ctx->d_order + gc, inverse.data(), (size_t)gc * 4, hipMemcpyHostToDevice));
        }
        hipEvent_t ev1 = nullptr;
        MF_HIP(ctx, begin_launch_timing(ctx, &ev1));
        MF_HIP(ctx, mf::launch_sgd_ring(ctx->dtype, ctx->k, !hog, short_prefetch, ctx->lds_waves_used, false, nullptr, ctx->dP, ctx->dQt,
                                        ctx->dU, ctx->dV, ctx->dR, lsched.d_begin, lsched.d_len, lsched.d_hot, lsched.d_ring,
                                        ctx->part.gr, ctx->part.gc, lds_bytes, lr, lambda, ctx->d_ring_done,
                                        ctx->ring_epochs * ctx->part.gc, d_flags,
                                        (long long)ctx->spin_limit, stratum_order ? ctx->d_order : nullptr,
                                        stratum_order ? ctx->d_order + gc : nullptr, plan.packed ? plan.touched : nullptr,
                                        plan.touched_words, plan.slot_table_at, n_epochs, ctx->stream));
        if (ev1) MF_HIP(ctx, hipEventRecord(ev1, ctx->stream));
        ctx->ring_epochs += n_epochs;
        return MF_OK;
    }
    // Streamed mode: the ratings of a stratum are one contiguous piece of the packed arrays.  The
    // strata of `group` consecutive steps are copied from pinned host memory into one of two device
    // buffers on a second stream while the group before is computed (the overlap of transfer and
    // kernel of the paper's Section 5.3); groups keep a transfer above a few MiB, below which the
    // hand-off between the two streams costs more than the transfer.
    const int32_t gr_ = ctx->part.gr;
    const int32_t group = ctx->streamed ? ctx->stream_group : 1;
    auto stratum_range = [&](int32_t st, int64_t& begin, int64_t& size) {
        begin = ctx->part.block_ptr[(size_t)st * gr_];
        size = ctx->part.block_ptr[(size_t)(st + 1) * gr_] - begin;
    };
    auto stratum_of = [&](int32_t step) { return stratum_order ? stratum_order[step] : step; };
    auto enqueue_copy = [&](int32_t first_step, int buf) -> hipError_t {
        hipError_t e = hipSuccess;
        // the buffer's previous contents must have been used up by their kernels
        if (ctx->consumed_recorded[buf]) e = hipStreamWaitEvent(ctx->copy_stream, ctx->consumed[buf], 0);
        const int32_t last_step = std::min(gc, first_step + group);
        if (!stratum_order) {
            // natural order: the strata of the group are one piece of the host array
            int64_t begin, size, end_begin, end_size;
            stratum_range(first_step, begin, size);
            stratum_range(last_step - 1, end_begin, end_size);
            const int64_t total = end_begin + end_size - begin;
            if (e == hipSuccess && total > 0)
                e = hipMemcpyAsync(ctx->d_stream_buf[buf], ctx->h_packed + (size_t)begin * 12, (size_t)total * 12,
                                   hipMemcpyHostToDevice, ctx->copy_stream);
        } else {
            int64_t offset = 0;
            for (int32_t step = first_step; step < last_step && e == hipSuccess; ++step) {
                int64_t begin, size;
                stratum_range(stratum_of(step), begin, size);
                if (size > 0)
                    e = hipMemcpyAsync(ctx->d_stream_buf[buf] + (size_t)offset * 12, ctx->h_packed + (size_t)begin * 12,
                                       (size_t)size * 12, hipMemcpyHostToDevice, ctx->copy_stream);
                offset += size;
            }
        }
        if (e == hipSuccess) e = hipEventRecord(ctx->copied[buf], ctx->copy_stream);
        return e;
    };
    if (ctx->streamed && gc > 0) MF_HIP(ctx, enqueue_copy(0, 0));
    int64_t offset_in_buffer = 0;        // ratings of the group's earlier strata
    for (int32_t step = 0; step < gc; ++step) {
        const int32_t st = stratum_of(step);
        const int32_t* U = ctx->dU;
        const int32_t* V = ctx->dV;
        const float* R = ctx->dR;
        const int buf = (step / group) & 1;
        if (ctx->streamed) {
            if (step % group == 0) {
                if (step + group < gc) MF_HIP(ctx, enqueue_copy(step + group, buf ^ 1));
                MF_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->copied[buf], 0));
                offset_in_buffer = 0;
            }
            // the work lists hold positions in the packed order: shift the base so that position
            // `begin` of the packed order is the first element of this stratum's piece
            int64_t begin, size;
            stratum_range(st, begin, size);
            const char* piece = ctx->d_stream_buf[buf] + (size_t)offset_in_buffer * 12;
            U = (const int32_t*)piece - begin;
            V = (const int32_t*)(piece + (size_t)size * 4) - begin;
            R = (const float*)(piece + (size_t)size * 8) - begin;
            offset_in_buffer += size;
        }
        int64_t first, count;
        if (use_lds) {
            first = lsched.stratum_block[st];
            count = lsched.stratum_block[st + 1] - first;
        } else {
            first = s.stratum_entry[st];
            count = s.stratum_entry[st + 1] - first;
        }
        hipEvent_t ev1 = nullptr;
        if (count > 0) MF_HIP(ctx, begin_launch_timing(ctx, &ev1));
        if (count > 0 && use_lds)
            MF_HIP(ctx, mf::launch_sgd_lds(ctx->dtype, ctx->k, !hog, short_prefetch, ctx->lds_waves_used, ctx->dP, ctx->dQt, U, V,
                                           R, lsched.d_begin, lsched.d_len, lsched.d_hot, lsched.d_blocks + first, count, lds_bytes,
                                           lr, lambda, d_flags + 1, plan.packed ? plan.touched : nullptr,
                                           plan.touched_words, plan.slot_table_at, ctx->stream));
        else if (count > 0)
            MF_HIP(ctx, mf::launch_sgd(ctx->dtype, ctx->k, mode == MF_MODE_HOGWILD, ctx->dP, ctx->dQt, U, V, R,
                                       s.d_begin, s.d_len, first, count, lr, lambda, ctx->stream));
        if (ev1) MF_HIP(ctx, hipEventRecord(ev1, ctx->stream));
        if (ctx->streamed && ((step + 1) % group == 0 || step + 1 == gc)) {
            MF_HIP(ctx, hipEventRecord(ctx->consumed[buf], ctx->stream));
            ctx->consumed_recorded[buf] = true;
        }
    }
    return MF_OK;
}
}  // namespace

int mf_rmse(mf_ctx* ctx, const int32_t* d_rows, const int32_t* d_cols, const float* d_vals,
            int64_t count, double* rmse_out)
{
    if (!ctx || !rmse_out) return MF_EINVAL;
    if (!ctx->inited) return fail(ctx, MF_ESTATE, "mf_rmse before mf_init");
    if (!d_rows) {
        if (!ctx->loaded) return fail(ctx, MF_ESTATE, "no training ratings loaded");
        if (ctx->streamed) return fail(ctx, MF_ESTATE, "the training ratings are not resident on the device (streamed mode)");
        d_rows = ctx->dU;
        d_cols = ctx->dV;
        d_vals = ctx->dR;
        count = ctx->part.nnz;
    } else if (!d_cols || !d_vals) {
        return fail(ctx, MF_EINVAL, "null rating array");
    }
    if (count <= 0) return fail(ctx, MF_EINVAL, "RMSE over an empty set");
    MF_HIP(ctx, hipSetDevice(ctx->device));
    double* d_sum = ctx->d_partials + mf::kRmsePartials;
    MF_HIP(ctx, mf::launch_rmse(ctx->dtype, ctx->k, ctx->dP, ctx->dQt, d_rows, d_cols, d_vals, count,
                                ctx->d_partials, d_sum, false, ctx->stream));
    double sum = 0.0;
    MF_HIP(ctx, hipMemcpyAsync(&sum, d_sum, sizeof(double), hipMemcpyDeviceToHost, ctx->stream));
    MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    *rmse_out = std::sqrt(sum / (double)count);
    return check_device_flags(ctx);
}

int mf_rmse_noalloc(mf_ctx* ctx, const int32_t* d_rows, const int32_t* d_cols, const float* d_vals,
                    int64_t count, double* d_rmse_out)
{
    if (!ctx || !d_rmse_out) return MF_EINVAL;
    if (!ctx->inited) return fail(ctx, MF_ESTATE, "mf_rmse_noalloc before mf_init");
    if (!d_rows || !d_cols || !d_vals) return fail(ctx, MF_EINVAL, "null rating array");
    if (count <= 0) return fail(ctx, MF_EINVAL, "RMSE over an empty set");
    if (count > MF_RMSE_NOALLOC_MAX_COUNT)
        return fail(ctx, MF_EINVAL, "count exceeds MF_RMSE_NOALLOC_MAX_COUNT (2^32 entries)");
    if (ctx->device >= kMaxDevices || !g_scratch_addr[ctx->device])
        return fail(ctx, MF_EDEVICE, "no static scratch on this device (device index above 63)");
    MF_HIP(ctx, hipSetDevice(ctx->device));
    // every wavefront of the fixed launch shape writes its partial, so the scratch needs no
    // clearing although it still holds the previous call's values
    MF_HIP(ctx, mf::launch_rmse(ctx->dtype, ctx->k, ctx->dP, ctx->dQt, d_rows, d_cols, d_vals, count,
                                g_scratch_addr[ctx->device], d_rmse_out, true, ctx->stream));
    return MF_OK;
}

int mf_sync(mf_ctx* ctx)
{
    if (!ctx) return MF_EINVAL;
    MF_HIP(ctx, hipSetDevice(ctx->device));
    MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return check_device_flags(ctx);
}

int mf_profile_read(mf_ctx* ctx, double* kernel_ms_out, int64_t* launches_out)
{
    if (!ctx) return MF_EINVAL;
    MF_HIP(ctx, hipSetDevice(ctx->device));
    MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    // An event pair around nothing still measures the time between its two markers; take the
    // smallest of a few such empty pairs now and remove it from every bracketed launch.
    float empty_ms = 0.f;
    if (ctx->events_used > 0) {
        constexpr int kEmptyPairs = 16;
        hipEvent_t ev[2 * kEmptyPairs];
        for (auto& e : ev) MF_HIP(ctx, hipEventCreate(&e));
        for (auto& e : ev) MF_HIP(ctx, hipEventRecord(e, ctx->stream));
        MF_HIP(ctx, hipStreamSynchronize(ctx->stream));
        empty_ms = 1e30f;
        for (int i = 0; i < kEmptyPairs; ++i) {
            float ms = 0.f;
            MF_HIP(ctx, hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]));
            empty_ms = ms < empty_ms ? ms : empty_ms;
        }
        for (auto& e : ev) (void)hipEventDestroy(e);
    }
    double total = 0.0;
    for (size_t i = 0; i < ctx->events_used; ++i) {
        float ms = 0.f;
        MF_HIP(ctx, hipEventElapsedTime(&ms, ctx->events[i].first, ctx->events[i].second));
        total += ms > empty_ms ? ms - empty_ms : 0.f;
    }
    if (kernel_ms_out) *kernel_ms_out = total;
    if (launches_out) *launches_out = (int64_t)ctx->events_used;
    ctx->events_used = 0;
    return MF_OK;
}

int mf_debug_xcc_ids(mf_ctx* ctx, int32_t n_groups, int32_t* xcc_out)
{
    if (!ctx || !xcc_out) return MF_EINVAL;
    if (n_groups < 1 || n_groups > (1 << 20)) return fail(ctx, MF_EINVAL, "n_groups must be in [1, 2^20]");
    MF_HIP(ctx, hipSetDevice(ctx->device));
    int32_t* d = nullptr;
    MF_HIP(ctx, hipMalloc((void**)&d, (size_t)n_groups * 4));
    hipError_t e = mf::launch_xcc_probe(n_groups, d, ctx->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(xcc_out, d, (size_t)n_groups * 4, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    (void)hipFree(d);
    if (e != hipSuccess) return fail_hip(ctx, "xcc probe", e);
    return MF_OK;
}

int mf_suggest_grid(int64_t m, int64_t n, int64_t nnz, int32_t k, int32_t mode, int32_t* grid_r_out,
                    int32_t* grid_c_out, int32_t* split_out)
{
    if (m < 1 || n < 1 || nnz < 0 || !valid_k(k) || !grid_r_out || !grid_c_out || !split_out) return MF_EINVAL;
    if (mode != MF_MODE_DET && mode != MF_MODE_HOGWILD) return MF_EINVAL;
    const bool hog = mode == MF_MODE_HOGWILD;
    // few enough blocks for ~64 (Hogwild) / ~40 (deterministic) ratings in each; the deterministic
    // form, one wavefront per workgroup, wants many block rows (measured on 99 M ratings: 1.65 G
    // updates/s with 512, 2.10 G with 1024, no more with 2048)
    const double per_block = hog ? 64.0 : 40.0;
    int64_t g = (int64_t)std::floor(std::sqrt((double)std::max<int64_t>(nnz, 1) / per_block));
    g = std::min<int64_t>(g, hog ? 224 : 1024);
    g = std::max<int64_t>(g, 1);
    // LDS of a strip: all of a compute unit's for Hogwild; for the deterministic form the share that
    // lets g workgroups be resident on 256 compute units (half above 256 block rows, a quarter above 512)
    const int64_t lds = hog || g <= 256 ? (int64_t)mf::kLdsBudget : (g <= 512 ? 80 * 1024 - 1024 : 40 * 1024 - 1024);
    const int64_t strip_cols = std::max<int64_t>(1, lds / ((int64_t)k * 4));   // columns one strip may hold
    // enough column strips for the widest one (at most about 2*n/grid_c columns) to fit
    const int64_t gc_for_lds = (2 * n + strip_cols - 1) / strip_cols;
    int64_t gr = std::min<int64_t>(g, m);
    int64_t gc = std::min<int64_t>(std::max<int64_t>(g, gc_for_lds), n);
    gr = std::min(gr, gc);
    *grid_r_out = (int32_t)gr;
    *grid_c_out = (int32_t)gc;
    *split_out = MF_SPLIT_NNZ_WIDTH_BALANCED;
    return MF_OK;
}

int mf_plan_host(const int32_t* rows, const int32_t* cols, int64_t nnz, int64_t m, int64_t n,
                 int32_t grid_r, int32_t grid_c, int32_t split, int32_t mode, int32_t chunk,
                 int32_t xcd_affinity, int64_t* perm, int64_t* block_ptr, int32_t* row_bounds,
                 int32_t* col_bounds, int64_t* entry_begin, int32_t* entry_len, int64_t entry_cap,
                 int64_t* stratum_entry, int64_t* n_entries_out)
{
    if (check_grid(nullptr, nnz, grid_r, grid_c)) return MF_EINVAL;
    if (m < 1 || n < 1 || grid_r > m || grid_c > n) return MF_EINVAL;
    if (split < MF_SPLIT_EQUAL_WIDTH || split > MF_SPLIT_NNZ_WIDTH_BALANCED) return MF_EINVAL;
    if (mode != MF_MODE_DET && mode != MF_MODE_HOGWILD && mode != MF_PLAN_HOGWILD_LDS && mode != MF_PLAN_LDS_CUT_ROWS)
        return MF_EINVAL;
    if (chunk < 0 || (nnz > 0 && (!rows || !cols))) return MF_EINVAL;
    try {
        mf::Partition part;
        std::vector<int32_t> pu, pv;
        std::vector<float> pr, vals((size_t)nnz, 0.f);
        std::string err;
        int rc = mf::build_partition(rows, cols, vals.data(), nnz, m, n, grid_r, grid_c, split, 0, part, pu, pv, pr, err);
        if (rc) return rc;
        mf::RowStarts rs;
        mf::row_starts_from_rows(pu.data(), nnz, rs);
        mf::Schedule s;
        int64_t bound;
        if (mode == MF_MODE_DET) {
            mf::build_det_schedule(part, xcd_affinity != 0, s);
            bound = mf::det_entries_bound(grid_r, grid_c);
        } else if (mode == MF_MODE_HOGWILD) {
            mf::build_hogwild_schedule(part, rs, chunk, 16, xcd_affinity != 0, s);
            bound = mf::hogwild_entries_bound(nnz, grid_r, grid_c, chunk, 16);
        } else {
            mf::LdsSchedule l;
            mf::build_lds_schedule(part, rs, chunk, 16, mf::kMaxHotRows, l);
            if (mode == MF_PLAN_LDS_CUT_ROWS) {
                bound = mf::lds_hot_bound(nnz, grid_r, grid_c);
                s.begin = l.hot_pos;
                s.len.assign(l.hot_pos.size(), 0);
                s.stratum_entry.assign((size_t)grid_c + 1, 0);
                for (size_t L = 0; L < l.ring.size(); ++L)
                    for (int32_t j = 0; j < (l.ring[L].hot & 15); ++j) s.len[(size_t)(l.ring[L].hot >> 4) + j] = (int32_t)L;
            } else {
                bound = mf::lds_entries_bound(nnz, grid_r, grid_c, chunk, 16);
                s.begin = l.begin;
                s.len = l.len;
                s.stratum_entry.assign((size_t)grid_c + 1, (int64_t)l.begin.size());
                for (int32_t st = 0; st < grid_c; ++st)   // first entry of the first block of the stratum
                    if (l.stratum_block[st] < (int64_t)l.blocks.size())
                        s.stratum_entry[st] = l.blocks[(size_t)l.stratum_block[st]].first_entry;
            }
        }
        if ((int64_t)s.begin.size() > bound) return MF_ENOMEM;
        if (perm && nnz > 0) std::memcpy(perm, part.perm.data(), (size_t)nnz * 8);
        if (block_ptr) std::memcpy(block_ptr, part.block_ptr.data(), part.block_ptr.size() * 8);
        if (row_bounds) std::memcpy(row_bounds, part.row_bounds.data(), part.row_bounds.size() * 4);
        if (col_bounds) std::memcpy(col_bounds, part.col_bounds.data(), part.col_bounds.size() * 4);
        if (n_entries_out) *n_entries_out = (int64_t)s.begin.size();
        if (entry_begin || entry_len) {
            if ((int64_t)s.begin.size() > entry_cap) return MF_ENOMEM;
            if (entry_begin && !s.begin.empty()) std::memcpy(entry_begin, s.begin.data(), s.begin.size() * 8);
            if (entry_len && !s.len.empty()) std::memcpy(entry_len, s.len.data(), s.len.size() * 4);
        }
        if (stratum_entry) std::memcpy(stratum_entry, s.stratum_entry.data(), s.stratum_entry.size() * 8);
    } catch (const std::bad_alloc&) {
        return MF_ENOMEM;
    }
    return MF_OK;
}

}  // extern "C"
