// Internal declarations shared by the translation units of libmf_sgd (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <utility>
#include <vector>

namespace mf {

constexpr int kWave = 64;            // gfx950 wavefront width
constexpr int kWavesPerGroup = 4;    // 256 threads per workgroup
constexpr int kGroupThreads = kWave * kWavesPerGroup;
constexpr int kXcds = 8;             // accelerator dies of an MI355X; workgroup i is placed on die i mod 8
constexpr int kRmseGroups = 2048;    // fixed launch shape of the RMSE partial kernel
constexpr int kRmsePartials = kRmseGroups * kWavesPerGroup;

// One unit of work of a wavefront: `len` consecutive ratings of the packed order from `begin`.
struct Schedule {
    std::vector<int64_t> begin;          // per entry
    std::vector<int32_t> len;            // per entry (0 = padding, the wavefront exits at once);
                                         // sign bit set = the entry shares a row of P with others
    std::vector<int64_t> stratum_entry;  // first entry of stratum s (size G_c + 1)
    int64_t* d_begin = nullptr;          // device copies inside the caller's workspace
    int32_t* d_len = nullptr;
};

// Work of one workgroup of the LDS-resident Hogwild kernel: one block of the grid.  The block's
// strip of Qt (columns col0 .. col0+ncols) is held in LDS while the wavefronts of the workgroup
// take the block's entries (chunks of whole rows) one after another.
// Rows of P that the boundaries between the block's entries cut (very long rows shared out over
// several wavefronts) are held in LDS beside the strip while the block runs: `hot` = number of
// such rows (low 4 bits, at most kMaxHotRows) and the index of the first of them in the
// schedule's hot_pos list (the bits above).
// `id` = the block's linear id L = stratum * G_r + block row; it indexes the table of touched
// columns (one bit per column of the block's strip: set when the block has a rating there),
// with which the Hogwild LDS kernels keep only those columns in LDS, packed.
constexpr int32_t kMaxHotRows = 8;
constexpr int32_t kMaxTouchedWords = 64;   // bit words per block of that table (one per lane of a wavefront)
struct LdsBlock {
    int64_t first_entry;
    int32_t n_entries;
    int32_t col0;
    int32_t ncols;
    int32_t hot;
    int32_t id;
    int32_t reserved;
};

struct LdsSchedule {
    std::vector<int64_t> begin;          // per entry, block after block (no padding)
    std::vector<int32_t> len;            // per entry; sign bit = shares its row of P
    std::vector<LdsBlock> blocks;        // non-empty blocks, stratum after stratum
    std::vector<LdsBlock> ring;          // all G_c * G_r blocks, [stratum][block row], for the ring kernel
    std::vector<int64_t> stratum_block;  // first block of stratum s (size G_c + 1)
    std::vector<int64_t> hot_pos;        // per cut row of a block: the packed position of one of its ratings
    int32_t max_cols = 0;                // widest column strip of the grid
    int32_t max_hot = 0;                 // most cut rows any block keeps in LDS
    int64_t* d_begin = nullptr;
    int32_t* d_len = nullptr;
    LdsBlock* d_blocks = nullptr;
    LdsBlock* d_ring = nullptr;
    int64_t* d_hot = nullptr;
    uint32_t* d_touched = nullptr;       // touched-column bits, touched_words per block id; null = not built
    int32_t touched_words = 0;
};

// Where the runs of one matrix row begin in the packed order: bit i is set when rating i has
// another row index than rating i-1 (bit 0 always).  The schedule builders cut blocks there.
struct RowStarts {
    std::vector<uint64_t> bits;
    bool starts(int64_t i) const { return (bits[(size_t)(i >> 6)] >> (i & 63)) & 1; }
};
void row_starts_from_rows(const int32_t* pu, int64_t nnz, RowStarts& out);

// SplitMix64 output function (published algorithm): the counter-based source of every seeded
// choice of the library.
__host__ __device__ inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

// Seeded order of the rows inside a block (MF_OPT_ROW_ORDER_SEED): the rows of a row strip of
// `width` rows are visited in the order of (offset_in_strip * kRowOrderPrime + shift) mod width, an
// affine map with a prime multiplier above any width, hence a permutation of the strip's rows.
constexpr uint64_t kRowOrderPrime = 2147483647ULL;
__host__ __device__ inline uint32_t row_order_shift(uint64_t row_seed, int32_t a, int32_t width)
{
    return (uint32_t)(mix64(row_seed + (uint64_t)a) % (uint64_t)width);
}
__host__ __device__ inline uint32_t row_order_rank(uint32_t offset_in_strip, uint32_t shift, uint32_t width)
{
    return (uint32_t)(((uint64_t)offset_in_strip * kRowOrderPrime + shift) % width);
}

// Host partition of R into the block grid.
struct Partition {
    int64_t nnz = 0;
    int32_t gr = 0, gc = 0;
    std::vector<int64_t> perm;        // packed position -> original position (empty if kept on the device)
    std::vector<int64_t> block_ptr;   // gr*gc + 1
    std::vector<int32_t> row_bounds;  // gr + 1
    std::vector<int32_t> col_bounds;  // gc + 1
};

// partition.cpp ------------------------------------------------------------------------------
// Returns 0 or an MF_E* code; fills `out` and the packed COO arrays (host).
// row_seed != 0: rows of a block in the seeded order above instead of ascending.
int build_partition(const int32_t* rows, const int32_t* cols, const float* vals, int64_t nnz,
                    int64_t m, int64_t n, int32_t gr, int32_t gc, int32_t split, uint64_t row_seed, Partition& out,
                    std::vector<int32_t>& pu, std::vector<int32_t>& pv, std::vector<float>& pr,
                    std::string& err);
// Strip boundaries (size g + 1) of one axis: uniform division, or balanced by the per-id rating
// counts `degree` (see mf_sgd.h for the two balanced rules); strip index of every id.
void equal_width_bounds(int64_t size, int32_t g, std::vector<int32_t>& b);
void bounds_from_degrees(const int32_t* degree, int64_t nnz, int64_t size, int32_t g, bool width_weight,
                         std::vector<int32_t>& b);
void strip_table(const std::vector<int32_t>& bounds, int64_t size, std::vector<int32_t>& table);
// DET schedule: one entry per block.  HOGWILD schedule: blocks cut into chunks of whole rows.
void build_det_schedule(const Partition& part, bool xcd_affinity, Schedule& out);
void build_hogwild_schedule(const Partition& part, const RowStarts& rs, int32_t chunk,
                            int32_t waves, bool xcd_affinity, Schedule& out);
// hot_slots: how many cut rows a block may keep in LDS (0: none, they are updated in the L2).
void build_lds_schedule(const Partition& part, const RowStarts& rs, int32_t chunk,
                        int32_t waves, int32_t hot_slots, LdsSchedule& out);
// Deterministic mode on the LDS kernel: one entry (the whole block) per block descriptor.
void build_det_lds_schedule(const Partition& part, LdsSchedule& out);
// Upper bounds on the number of schedule entries, usable before the partition is known.
int64_t lds_entries_bound(int64_t nnz, int32_t gr, int32_t gc, int32_t chunk, int32_t waves);
int64_t lds_hot_bound(int64_t nnz, int32_t gr, int32_t gc);
int32_t widest_strip(const Partition& part);   // columns of the widest column strip
int64_t det_entries_bound(int32_t gr, int32_t gc);
int64_t hogwild_entries_bound(int64_t nnz, int32_t gr, int32_t gc, int32_t chunk, int32_t waves);

// partition_device.hip ------------------------------------------------------------------------
// The same partition computed on the device from COO arrays that already live in HBM: fills
// dU, dV, dR (packed order), d_perm (packed position -> original position; out.perm stays
// empty), the rest of `out`, and `rs` for the schedule builders.  Temporary device memory (about
// 24 bytes per rating) is allocated and freed inside.  Bit-identical to build_partition.
int build_partition_device(const int32_t* d_rows, const int32_t* d_cols, const float* d_vals, int64_t nnz,
                           int64_t m, int64_t n, int32_t gr, int32_t gc, int32_t split, uint64_t row_seed,
                           int32_t* dU, int32_t* dV, float* dR, uint32_t* d_perm, Partition& out, RowStarts& rs,
                           hipStream_t stream, std::string& err);

// kernels.hip ---------------------------------------------------------------------------------
hipError_t launch_sgd(int dtype, int k, bool hogwild, void* P, void* Qt, const int32_t* U,
                      const int32_t* V, const float* R, const int64_t* entry_begin,
                      const int32_t* entry_len, int64_t first_entry, int64_t n_entries, float lr,
                      float lambda, hipStream_t stream);
// LDS-resident kernel: one workgroup per block descriptor; `exact` = deterministic mode (one
// wavefront per workgroup, fp32 strip), else Hogwild (`waves` wavefronts, fixed-point strip;
// short_prefetch: rows of P are requested 4 instead of 8 ratings ahead, which pays when P is
// served from the caches).  hot_pos: the schedule's list of cut rows (see LdsBlock); lds_bytes
// covers the widest strip plus the most cut rows of any block.  range_flag (device): set to 1 by
// the Hogwild kernel when a value leaves the safe range of its fixed-point strip.
// touched (device, may be null) / touched_words / slot_table_at: the table of touched columns per
// block id (launch_mark_touched).  With it the Hogwild form keeps only the touched columns of a
// strip in LDS, packed; lds_bytes then covers the most touched columns of any block plus its cut
// rows, followed -- from the 32-bit word slot_table_at on -- by 64 bytes per bit word for the
// kernel's column -> slot table.
hipError_t launch_sgd_lds(int dtype, int k, bool exact, bool short_prefetch, int waves, void* P, void* Qt, const int32_t* U,
                          const int32_t* V, const float* R, const int64_t* entry_begin,
                          const int32_t* entry_len, const int64_t* hot_pos, const LdsBlock* blocks, int64_t n_blocks,
                          size_t lds_bytes, float lr, float lambda, int* range_flag, const uint32_t* touched,
                          int touched_words, int slot_table_at, hipStream_t stream);
// One launch per epoch (ring of workgroups, see kernels.hip).  ring_blocks: grid_c * grid_r
// descriptors indexed [stratum][block row], empty blocks included.  order / pos (device, grid_c
// entries each, both or neither): the stratum of every step and its inverse.  abort_flag: two
// device ints, [0] raised when a bounded wait expires, [1] the range flag.  query_only: do not launch,
// return in *max_resident how many workgroups of this shape the device can hold at once.
// touched / touched_words / slot_table_at: as for launch_sgd_lds.  n_epochs: epochs run by the one
// launch (more than one only with the strata in natural order); the caller then adds
// n_epochs * grid_c to `first` for the next launch.
hipError_t launch_sgd_ring(int dtype, int k, bool exact, bool short_prefetch, int waves, bool query_only, int* max_resident,
                           void* P, void* Qt, const int32_t* U, const int32_t* V, const float* R,
                           const int64_t* entry_begin, const int32_t* entry_len, const int64_t* hot_pos, const LdsBlock* ring_blocks,
                           int grid_r, int grid_c, size_t lds_bytes, float lr, float lambda, int* done,
                           int first, int* abort_flag, long long spin_limit, const int32_t* order,
                           const int32_t* pos, const uint32_t* touched, int touched_words, int slot_table_at,
                           int n_epochs, hipStream_t stream);
// Fill the table of touched columns for a list of blocks made for this call: first_entry = the
// block's first packed position, n_entries = its number of ratings, col0 / ncols / id as usual
// (rows of the table of blocks not in the list are left as they are: clear the table first).
// totals (device, three 64-bit counters, cleared by the caller): [0] += touched columns, [1] +=
// strip columns, summed over the blocks; [2] = the most touched columns of any block.
hipError_t launch_mark_touched(const LdsBlock* blocks, int64_t n_blocks, const int32_t* V, uint32_t* touched, int words,
                               unsigned long long* totals, hipStream_t stream);
size_t lds_strip_bytes(int k, int32_t max_cols);   // dynamic LDS the kernel needs for a grid
constexpr size_t kLdsBudget = 160 * 1024 - 1024;   // LDS of one gfx950 compute unit, minus static use
hipError_t launch_init(int dtype, void* X, int64_t count, uint64_t seed, uint64_t stream_id,
                       float scale, hipStream_t stream);
// partials: kRmsePartials doubles of device scratch (every one is overwritten).  root = false:
// *sum_out = the sum of squared errors; true: the root of their mean.
hipError_t launch_rmse(int dtype, int k, const void* P, const void* Qt, const int32_t* U,
                       const int32_t* V, const float* R, int64_t count, double* partials,
                       double* sum_out, bool root, hipStream_t stream);
hipError_t launch_xcc_probe(int32_t n_groups, int32_t* d_out, hipStream_t stream);
hipError_t launch_fill_i32(int32_t* d_out, int64_t count, int32_t value, hipStream_t stream);

}  // namespace mf
