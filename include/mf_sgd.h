/*
 * mf_sgd.h -- C ABI of the MI355X (gfx950) SGD matrix-factorization library.
 *
 * The library runs the training phase of the paper's Algorithm 1 ("SGD") -- for every rating
 * r_uv:  e = r_uv - p_u.q_v ;  p_u += lr*(e*q_v - lambda*p_u) ;  q_v += lr*(e*p_u - lambda*q_v),
 * both right-hand sides using the values read before the step -- over a grid of blocks of the
 * sparse rating matrix R (m x n), on dense factors P (m x k) and Q (k x n), one epoch (every
 * rating exactly once) per call, on one GPU.  Blocks that share neither a row strip nor a column
 * strip are independent (Section 3.1, Example 2) and are processed concurrently.
 *
 * Conventions
 *   - No exception crosses this boundary; no call aborts or prints.  Every call returns an int:
 *     MF_OK or a negative MF_E* code; mf_last_error() gives a message for the last failure.
 *   - "host" / "device" is stated for every pointer.  Device pointers are plain HIP device
 *     addresses (for instance torch tensors' data_ptr()).  The caller owns every buffer it
 *     passes; the library owns its context, its host-side metadata, one small device buffer
 *     for reduction partials (allocated in mf_create, freed in mf_destroy), the temporary device
 *     memory of mf_load_blocks_device (freed before it returns) and, in streamed mode only, the
 *     pinned host copy of the ratings and two device buffers (freed by the next load or by
 *     mf_destroy).
 *   - Indices are 0-based.  Q is held transposed: Qt is n x k row-major and Qt[v] is the
 *     paper's column q_v.  P is m x k row-major.
 *   - A context is not thread-safe.  All device work is enqueued on the stream given to
 *     mf_create; calls that return data to the host synchronise that stream.
 */
#ifndef MF_SGD_H
#define MF_SGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mf_ctx mf_ctx;

enum {
    MF_OK = 0,
    MF_EINVAL = -1,   /* bad argument                                   */
    MF_ESTATE = -2,   /* call out of order (e.g. epoch before load)     */
    MF_ENOMEM = -3,   /* workspace too small / host allocation failed   */
    MF_EDEVICE = -4,  /* a HIP call failed, or the one-launch kernel gave up a wait */
    MF_ERANGE = -5    /* a row / column index outside [0,m) / [0,n); or a factor  */
                      /* left the range of the Hogwild kernel's fixed-point strip */
};

enum { MF_F32 = 0, MF_F16 = 1 };               /* storage type of the factors; arithmetic is fp32 */
enum { MF_MODE_DET = 0, MF_MODE_HOGWILD = 1 };
enum { MF_SPLIT_EQUAL_WIDTH = 0, MF_SPLIT_NNZ_BALANCED = 1, MF_SPLIT_NNZ_WIDTH_BALANCED = 2 };

/* Tuning options for mf_set_option (all have working defaults). */
enum {
    MF_OPT_HOGWILD_CHUNK = 1,     /* target ratings per wavefront of the L2-atomics Hogwild kernel;   */
                                  /* 0 (default) = the block's ratings divided by MF_OPT_LDS_WAVES,   */
                                  /* which bounds how many wavefronts change one column concurrently */
    MF_OPT_XCD_AFFINITY = 2,      /* 1 (default): all wavefronts working on one block are placed on  */
                                  /* one XCD; 0: spread over all XCDs                                 */
    MF_OPT_PROFILE = 3,           /* 1: time every SGD kernel launch with HIP events (see below)     */
    MF_OPT_HOGWILD_KERNEL = 4,    /* MF_HOGWILD_AUTO (default), _GLOBAL_ATOMICS or _LDS, see          */
                                  /* mf_sgd_epoch                                                     */
    MF_OPT_LDS_CHUNK = 5,         /* target ratings per work-list entry of the LDS kernel; 0 (default)*/
                                  /* = the smallest cap on an entry's ratings with which a block      */
                                  /* gives at most MF_OPT_LDS_WAVES entries                           */
    MF_OPT_LDS_WAVES = 6,         /* wavefronts per workgroup of the LDS kernel, 1..16.  Default:     */
                                  /* chosen by mf_load_blocks -- one per eight ratings of an average  */
                                  /* block, between 4 and 16                                          */
    MF_OPT_DET_KERNEL = 7,        /* MF_KERNEL_AUTO (default), _GLOBAL or _LDS for MF_MODE_DET        */
    MF_OPT_RING = 8,              /* 1 (default): with the LDS kernels, run an epoch as ONE launch in */
                                  /* which the workgroups hand the column strips round (see           */
                                  /* mf_sgd_epoch) when all grid_r workgroups fit the device at once; */
                                  /* 0: always one launch per stratum                                 */
    MF_OPT_RING_SPIN_LIMIT = 9,   /* polls after which a waiting workgroup gives up (default 2^22)    */
    MF_OPT_LDS_PREFETCH = 10,     /* MF_MODE_HOGWILD, LDS kernels: rows of P requested ahead.  4 = the */
                                  /* short depth (4 ratings), 8 = the long one (8 ratings, 12 with    */
                                  /* binary16 storage); 0 (default): short if P takes at most 64 MiB  */
    MF_OPT_PACK_STRIPS = 12,      /* read by mf_load_blocks(_device): 1 (default) = the LDS kernels   */
                                  /* keep only the touched columns of a strip in LDS where that pays  */
                                  /* or whole strips do not fit (see mf_sgd_epoch); 2 = wherever the  */
                                  /* packed form is possible; 0 = always whole strips                 */
    MF_OPT_ROW_ORDER_SEED = 11    /* read by mf_load_blocks(_device): 0 (default) = the rows of a     */
                                  /* block in ascending order; else they are visited in a seeded      */
                                  /* order (the paper's scheduler visits "randomly", Section 3.1):    */
                                  /* rows of row strip a by ((u - first) * 2147483647 + shift_a) mod  */
                                  /* width, shift_a = mix(seed + a) mod width, mix = the SplitMix64   */
                                  /* output function.  The ratings of a row stay together.            */
};
enum { MF_KERNEL_AUTO = 0, MF_KERNEL_GLOBAL = 1, MF_KERNEL_LDS = 2 };
enum { MF_HOGWILD_AUTO = MF_KERNEL_AUTO, MF_HOGWILD_GLOBAL_ATOMICS = MF_KERNEL_GLOBAL, MF_HOGWILD_LDS = MF_KERNEL_LDS };
enum { MF_PLAN_HOGWILD_LDS = 2, MF_PLAN_LDS_CUT_ROWS = 3 };  /* values of `mode` accepted by mf_plan_host only */
enum { MF_KERNEL_ID_CHUNKS = 1, MF_KERNEL_ID_BLOCK_LDS = 2, MF_KERNEL_ID_RING_LDS = 3 };  /* see mf_epoch_plan */

/* Create a context on HIP device `device`.  `hip_stream` is a hipStream_t of the caller (may be
 * NULL for the default stream); all work of this context is enqueued on it. */
int mf_create(mf_ctx** out, int device, void* hip_stream);
int mf_destroy(mf_ctx* ctx);

/* Message of the last failed call on ctx (owned by ctx, valid until the next call on ctx). */
const char* mf_last_error(const mf_ctx* ctx);

/* Set a tuning option.  Must be called before mf_load_blocks to affect the schedule. */
int mf_set_option(mf_ctx* ctx, int32_t option, int64_t value);

/* "init_model" of Algorithm 1.  Registers the factor buffers and optionally fills them.
 *   m, n      : size of R;  k : number of latent factors, one of 32, 64, 128, 256.
 *   dtype     : MF_F32 or MF_F16 -- element type of dP and dQt.
 *   dP        : DEVICE, m*k elements, row-major, caller-owned, 16-byte aligned.
 *   dQt       : DEVICE, n*k elements, row-major, caller-owned, 16-byte aligned.
 *   scale >= 0: every element i of P becomes scale*U(seed,0,i), of Qt scale*U(seed,1,i), where
 *               U is a counter-based uniform generator on the 24-bit grid in [0,1) (the paper
 *               only says the factors start from random values); in MF_F16 the value is rounded
 *               to binary16 (nearest even).
 *   scale < 0 : the buffers keep their current contents (the caller initialised them).
 * The buffers stay registered (and are updated in place by mf_sgd_epoch) until the next mf_init. */
int mf_init(mf_ctx* ctx, int64_t m, int64_t n, int32_t k, int32_t dtype,
            void* dP, void* dQt, uint64_t seed, float scale);

/* Size in bytes of the device workspace mf_load_blocks needs for nnz ratings on this grid. */
int mf_load_blocks_workspace(const mf_ctx* ctx, int64_t nnz, int32_t grid_r, int32_t grid_c,
                             size_t* bytes_out);

/* Partition R into a grid_r x grid_c grid of blocks (Section 3.1) and upload it.
 *   rows, cols, vals : HOST arrays of nnz entries (COO triples, the paper's "triadic tuples"),
 *                      read-only, not retained.  Duplicate (u,v) entries are legal.
 *   grid_r <= grid_c, grid_r <= m, grid_c <= n.
 *   split            : MF_SPLIT_EQUAL_WIDTH  -- strip a = [ceil(a*size/G), ceil((a+1)*size/G)) (the
 *                                               uniform division);
 *                      MF_SPLIT_NNZ_BALANCED -- strip bounds chosen so that every strip holds about
 *                                               nnz/G ratings: bounds[a] = the smallest id whose
 *                                               exclusive degree prefix is >= ceil(a*nnz/G).
 *                      MF_SPLIT_NNZ_WIDTH_BALANCED -- every id x weighs deg(x)*size + nnz (its share
 *                                               of the ratings plus its share of the axis); with the
 *                                               exclusive prefix W[x] = S[x]*size + x*nnz, bounds[a]
 *                                               = the smallest x with W[x] >= ceil(a*2*nnz*size/G).
 *                                               No strip holds more than about 2*nnz/G ratings nor
 *                                               spans more than about 2*size/G ids, which bounds
 *                                               the LDS the Hogwild kernel needs per strip.
 *   d_workspace      : DEVICE, caller-owned, workspace_bytes >= mf_load_blocks_workspace(); must
 *                      stay alive and untouched until the next mf_load_blocks / mf_destroy.
 * Block (a,b) belongs to stratum s = (b-a) mod grid_c and has linear id L = s*grid_r + a; the
 * grid_r blocks of one stratum are mutually independent.  Ratings are stored block after block in
 * ascending L, inside a block in ascending (row, column, original position).
 * Requires mf_init first (m and n come from there).  Synchronises the stream. */
int mf_load_blocks(mf_ctx* ctx, const int32_t* rows, const int32_t* cols, const float* vals,
                   int64_t nnz, int32_t grid_r, int32_t grid_c, int32_t split,
                   void* d_workspace, size_t workspace_bytes);

/* mf_load_blocks for rating matrices that should NOT be kept in device memory: the packed ratings stay
 * in pinned host memory owned by the library (12 bytes per rating) and every epoch streams them to the
 * device stratum by stratum -- a stratum is one contiguous piece of the packed order; small strata
 * travel several at a time, about 4 MiB per transfer -- into two library-owned device buffers, on a
 * second stream of default priority, while the strata before are being computed (the overlap of
 * transfer and kernel that the paper's Section 5.3 describes for its GPU workers).  The workspace
 * (query its size with mf_load_blocks_streamed_workspace) holds the work lists only.  Epochs run one launch per stratum;
 * their results are those of mf_load_blocks with MF_OPT_RING = 0 (bit for bit in MF_MODE_DET).
 * mf_rmse over the training ratings (NULL arrays) is not available in this mode (MF_ESTATE).
 * rows, cols, vals: HOST pointers as for mf_load_blocks.  Errors as mf_load_blocks. */
int mf_load_blocks_streamed_workspace(const mf_ctx* ctx, int64_t nnz, int32_t grid_r, int32_t grid_c,
                                      size_t* bytes_out);
int mf_load_blocks_streamed(mf_ctx* ctx, const int32_t* rows, const int32_t* cols, const float* vals,
                            int64_t nnz, int32_t grid_r, int32_t grid_c, int32_t split, void* d_workspace,
                            size_t workspace_bytes);

/* mf_load_blocks for COO arrays that already live in device memory ("partition R" and
 * "preprocess data" of the paper's Algorithm 2, done on the GPU): the same partition, packed order
 * and work lists as mf_load_blocks, bit for bit, with the block ids, the sort and the gather
 * computed by kernels on the context's stream.  d_rows, d_cols, d_vals: DEVICE pointers, nnz entries
 * each, read only, not needed after the call returns.  d_workspace as for mf_load_blocks.  The call
 * allocates about 24 bytes per rating of temporary device memory (hipMalloc) and frees it before it
 * returns; it synchronises the stream.  Errors as mf_load_blocks, plus MF_EINVAL if block id, row
 * offset and column offset of the grid do not fit 64 key bits together (then use mf_load_blocks). */
int mf_load_blocks_device(mf_ctx* ctx, const int32_t* d_rows, const int32_t* d_cols, const float* d_vals,
                          int64_t nnz, int32_t grid_r, int32_t grid_c, int32_t split, void* d_workspace,
                          size_t workspace_bytes);

/* Copy the partition to HOST arrays of the caller (any pointer may be NULL):
 *   perm[nnz]                 original position of the rating stored at each packed position;
 *   block_ptr[grid_r*grid_c+1] start of every block in the packed order;
 *   row_bounds[grid_r+1], col_bounds[grid_c+1]. */
int mf_get_partition(const mf_ctx* ctx, int64_t* perm, int64_t* block_ptr,
                     int32_t* row_bounds, int32_t* col_bounds);

/* One epoch of Algorithm 1's training phase: every loaded rating exactly once, stratum after
 * stratum, on the context's stream (one kernel launch per stratum, or one per epoch, see
 * MF_OPT_RING below).  Returns after enqueueing.
 *   MF_MODE_DET     : one wavefront per block, ratings in stored order.  The result is the same
 *                     on every run and equals the sequential order (strata ascending, blocks
 *                     ascending, stored order) up to fp32 rounding.  Two kernels with identical
 *                     results: MF_KERNEL_LDS keeps the block's strip of Qt in LDS (fp32; taken by
 *                     MF_KERNEL_AUTO when a strip needs no more than the share of a compute
 *                     unit's 159 KiB of LDS that lets all grid_r single-wavefront workgroups be
 *                     resident: all of it up to 256 block rows, half up to 512, else a quarter),
 *                     MF_KERNEL_GLOBAL works on Qt in memory (any grid).
 *   MF_MODE_HOGWILD : every block is cut into chunks of whole rows that many wavefronts process
 *                     concurrently without locks (lock-free updates in the sense of Hogwild,
 *                     Section 3.1).  A wavefront owns the rows of P of its chunk; rows of Qt are
 *                     shared: each wavefront ADDS its change of q_v with an atomic operation,
 *                     computed from a value that other wavefronts may have changed meanwhile, so
 *                     no update is lost but the result varies from run to run.  Two kernels:
 *                       MF_HOGWILD_LDS            one workgroup per block keeps the block's strip
 *                                                 of Qt in LDS as 32-bit fixed point with 24
 *                                                 fraction bits and changes it with integer LDS
 *                                                 atomics (floating-point ones are some twenty
 *                                                 times slower on this chip).  While this kernel
 *                                                 is used the values of Qt are multiples of 2^-24
 *                                                 (the fp32 spacing in [0.5, 1)) and saturate at
 *                                                 +-128.  Needs (widest column strip) * k * 4
 *                                                 bytes <= 159 KiB of LDS -- or, with resident
 *                                                 ratings, only (most columns of a strip in
 *                                                 which one block has a rating) * k * 4 bytes:
 *                                                 when the blocks touch at most three quarters
 *                                                 of their strips' columns, or whole strips do
 *                                                 not fit, the kernel keeps just the touched
 *                                                 columns in LDS (a table made by the load call
 *                                                 says which; strips of up to 65536 / (k *
 *                                                 sizeof(element) / 4) columns).  A block's
 *                                                 ratings are divided over the wavefronts as
 *                                                 evenly as whole matrix rows allow; a row so
 *                                                 long that its share of a block is dealt to
 *                                                 several wavefronts has its p_u kept in LDS
 *                                                 in the same format while that block runs (up
 *                                                 to 8 such rows per block, as room beside
 *                                                 the strip allows; a block is never cut into
 *                                                 more pieces than that permits);
 *                       MF_HOGWILD_GLOBAL_ATOMICS wavefronts of a whole die share a block and use
 *                                                 floating-point atomics in that die's L2 (any
 *                                                 grid, slower).
 *                     MF_HOGWILD_AUTO takes the LDS kernel whenever the grid allows it.
 * With the LDS kernels and MF_OPT_RING = 1 the epoch is a single launch: workgroup a keeps block
 * row a, walks the strata in order and waits (bounded) for the workgroup that used its next column
 * strip last.  The order of the steps, and in MF_MODE_DET every bit of the result, is the same as
 * with one launch per stratum.  That kernel needs all grid_r workgroups on the device at the same
 * time: it is taken only when an otherwise idle device holds them, and the device should not be
 * shared while it runs.  If a wait exceeds its limit (MF_OPT_RING_SPIN_LIMIT) all workgroups leave
 * the kernel, the epoch is abandoned half-applied, the next mf_sync / mf_rmse returns MF_EDEVICE
 * once, and later epochs on this load run one launch per stratum, which needs no co-residency.
 * Divergence: MF_HOGWILD_LDS watches its fixed-point strip; when it reads a value of magnitude >= 64
 * or makes a single change of magnitude >= 4 (both far outside honest training; beyond +-128 a
 * strip word would wrap round) the next mf_sync / mf_rmse returns MF_ERANGE once; the factors are
 * then meaningless. */
int mf_sgd_epoch(mf_ctx* ctx, float lr, float lambda, int32_t mode);

/* What mf_sgd_epoch(mode) launches for the loaded grid, decided exactly as the epoch call decides it
 * (the choice depends on the grid: strips that do not fit the LDS, or more block rows than the device
 * holds workgroups at once, fall back to slower kernels, and a grid made for MF_MODE_HOGWILD is
 * usually a poor one for MF_MODE_DET).  Outputs are HOST pointers, any may be NULL:
 *   kernel_out   MF_KERNEL_ID_CHUNKS    one wavefront per work-list entry, Qt in memory, one launch per
 *                                       non-empty stratum;
 *                MF_KERNEL_ID_BLOCK_LDS one workgroup per block, the strip of Qt in LDS, one launch per
 *                                       non-empty stratum;
 *                MF_KERNEL_ID_RING_LDS  the same, one launch per epoch;
 *   launches_out kernel launches per epoch;   waves_out wavefronts per workgroup.
 * On success mf_last_error() returns a one-line description of the choice and, when a faster kernel
 * was not taken, the reason.  MF_ESTATE before mf_load_blocks. */
int mf_epoch_plan(mf_ctx* ctx, int32_t mode, int32_t* kernel_out, int64_t* launches_out, int32_t* waves_out);

/* One epoch with the strata visited in a given order (the paper's scheduler hands blocks out
 * "randomly", Section 3.1; Example 3 argues for balanced, random visiting): stratum_order is a HOST
 * array of grid_c numbers, a permutation of 0 .. grid_c-1, stratum_order[t] = stratum of step t;
 * NULL = natural order (then the call is mf_sgd_epoch).  Every rating is still visited exactly
 * once, blocks of a stratum and ratings of a block as in mf_sgd_epoch; MF_MODE_DET stays
 * deterministic.  With an order given, the call waits for the stream's earlier work before it
 * uploads the order.  MF_EINVAL if stratum_order is not a permutation. */
int mf_sgd_epoch_ordered(mf_ctx* ctx, float lr, float lambda, int32_t mode, const int32_t* stratum_order);

/* n_epochs epochs of mf_sgd_epoch(ctx, lr, lambda, mode), strata in natural order (Algorithm 1, the
 * training phase repeated).  Where an epoch is one launch (see mf_epoch_plan) the epochs run in ONE
 * launch: a block row goes on with the next epoch as soon as the strips it needs are free, instead
 * of waiting until every block row has finished the epoch, which in MF_MODE_DET is most of an
 * epoch's time on matrices with very popular columns.  The result is that of n_epochs calls of
 * mf_sgd_epoch (MF_MODE_DET: bit for bit).  n_epochs: 1 .. 4096, n_epochs * grid_c at most 2^29.
 * Errors as mf_sgd_epoch. */
int mf_sgd_epochs(mf_ctx* ctx, float lr, float lambda, int32_t mode, int32_t n_epochs);

/* Host-only: the per-epoch stratum permutation this library proposes (a convention, the paper
 * names no generator): stratum s gets the key mix(mix(seed ^ epoch * 0xD1B54A32D192ED03) + s) with
 * mix = the SplitMix64 output function, strata in ascending (key, s).  order_out: HOST, grid_c
 * numbers. */
int mf_stratum_order(uint64_t seed, uint64_t epoch, int32_t grid_c, int32_t* order_out);

/* RMSE = sqrt(mean (r - p_u.q_v)^2) of the current factors (the quality metric of Section 7).
 *   d_rows, d_cols, d_vals : DEVICE arrays of `count` entries, caller-owned; if d_rows is NULL
 *                            the loaded training ratings are used and count is ignored.
 *   rmse_out               : HOST.  Products and sums are taken in double; the reduction order is
 *                            fixed, so the value is reproducible.
 * count == 0 gives MF_EINVAL.  Synchronises the stream. */
int mf_rmse(mf_ctx* ctx, const int32_t* d_rows, const int32_t* d_cols, const float* d_vals,
            int64_t count, double* rmse_out);

/* mf_rmse for callers that cannot allocate device memory or wait (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same kernels and the same fixed-order
 * reduction, but the partial sums go to a static device array of the library (64 KiB per GPU, held
 * until the process ends) instead of the buffer mf_create allocates, the result
 * sqrt(mean (r - p_u.q_v)^2) is written to DEVICE memory of the caller, and the call neither
 * allocates, frees, copies to the host nor synchronises: it only enqueues two kernels on the
 * context's stream.
 *   d_rows, d_cols, d_vals : DEVICE arrays of `count` entries, caller-owned, all required;
 *   count                  : 1 .. MF_RMSE_NOALLOC_MAX_COUNT, else MF_EINVAL;
 *   d_rmse_out             : DEVICE, one double, valid once the stream has reached the call.
 * All calls on one GPU share that GPU's array (every call overwrites all of it, nothing has to be
 * cleared): calls that overlap in time on one GPU -- from two contexts, or from two streams -- race
 * and must be ordered by the caller.  Only devices 0..63 have the array (MF_EDEVICE above). */
#define MF_RMSE_NOALLOC_MAX_COUNT ((int64_t)1 << 32)
int mf_rmse_noalloc(mf_ctx* ctx, const int32_t* d_rows, const int32_t* d_cols, const float* d_vals,
                    int64_t count, double* d_rmse_out);

/* Wait for all work enqueued by this context. */
int mf_sync(mf_ctx* ctx);

/* With MF_OPT_PROFILE = 1 every SGD kernel launch is bracketed by HIP events on the context's
 * stream.  This call synchronises, then returns the summed kernel time in milliseconds and the
 * number of launches since the previous call (HOST pointers, either may be NULL).  Each bracket is
 * reduced by the duration of an empty event pair measured during this call, so that the figure
 * is the kernels' own time. */
int mf_profile_read(mf_ctx* ctx, double* kernel_ms_out, int64_t* launches_out);

/* Diagnostic: launch n_groups workgroups and report, for each, the id of the XCD (accelerator
 * die) it ran on.  xcc_out: HOST array of n_groups int32.  Used to check the workgroup-to-XCD
 * placement MF_OPT_XCD_AFFINITY relies on. */
int mf_debug_xcc_ids(mf_ctx* ctx, int32_t n_groups, int32_t* xcc_out);

/* Host-only: a grid and split rule for mf_load_blocks that suit the kernels of `mode` on an MI355X,
 * from the measured trade-off between the fixed cost of a stratum and the number of workgroups
 * that work at a time (the role the paper gives its kernel cost model, Section 5.3: block sizes
 * that are too small leave the GPU idle).  Rules: MF_MODE_HOGWILD wants about 224 x 224 blocks (all
 * block rows resident for the one-launch ring kernel), at least ~64 ratings per block, and column
 * strips that fit the LDS under MF_SPLIT_NNZ_WIDTH_BALANCED (at most 2*n/grid_c columns of k fp32
 * values in 159 KiB), which raises grid_c for wide matrices; MF_MODE_DET wants about 40 ratings per
 * block, up to 1024 block rows, and strips of the LDS share that keeps all of them resident (all of
 * it up to 256 block rows, half up to 512, else a quarter).  The grids are safe for any data of
 * that shape; where blocks touch few of their strips' columns, coarser grid_c may run faster (see
 * mf_sgd_epoch on packed strips; mf_epoch_plan tells what a grid gets).  All outputs are HOST
 * pointers. */
int mf_suggest_grid(int64_t m, int64_t n, int64_t nnz, int32_t k, int32_t mode,
                    int32_t* grid_r_out, int32_t* grid_c_out, int32_t* split_out);

/* Host-only planning (no device, no context): the partition mf_load_blocks would build for these
 * arguments, and the per-wavefront work list of one epoch mode, for inspection and for checking
 * the block rule of Section 3.1 without a GPU.  All pointers are HOST; any output may be NULL.
 *   perm, block_ptr, row_bounds, col_bounds : as in mf_get_partition.
 *   entry_begin[entry_cap], entry_len[entry_cap] : work-list entries (first packed position and
 *       number of ratings; length 0 = padding; in HOGWILD lists the sign bit of the length marks
 *       a piece of a matrix row that was cut because it is longer than two chunks, the low 31
 *       bits are the length); entry e of a stratum is run by workgroup e/4 of that stratum's
 *       launch, and with xcd_affinity = 1 workgroup w serves die w mod 8.
 *   stratum_entry[grid_c+1] : first entry of each stratum;  n_entries_out : entries in total.
 * mode = MF_PLAN_HOGWILD_LDS gives the work list of the LDS kernel: entries block after block
 * without padding (chunk = MF_OPT_LDS_CHUNK's meaning); every block's entries are taken by the
 * wavefronts of one workgroup.
 * mode = MF_PLAN_LDS_CUT_ROWS lists, for the same work list, the matrix rows that a boundary
 * between two entries of a block cuts (the LDS kernel keeps their p_u in LDS while the block runs;
 * a block whose even division would cut more than 8 rows is divided into fewer, longer chunks
 * until it cuts at most 8): entry_begin[i] = packed
 * position of one rating of the row, entry_len[i] = stratum * grid_r + block row of the block;
 * stratum_entry is zero-filled.
 * MF_ENOMEM if entry_cap is too small. */
int mf_plan_host(const int32_t* rows, const int32_t* cols, int64_t nnz, int64_t m, int64_t n,
                 int32_t grid_r, int32_t grid_c, int32_t split, int32_t mode, int32_t chunk,
                 int32_t xcd_affinity, int64_t* perm, int64_t* block_ptr, int32_t* row_bounds,
                 int32_t* col_bounds, int64_t* entry_begin, int32_t* entry_len, int64_t entry_cap,
                 int64_t* stratum_entry, int64_t* n_entries_out);

#ifdef __cplusplus
}
#endif
#endif /* MF_SGD_H */
