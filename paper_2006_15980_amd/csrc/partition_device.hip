// Device side of mf_load_blocks_device: the partition of the rating matrix into the block grid
// (Section 3.1 of the paper; "partition R" and "preprocess data" of its Algorithm 2) computed
// on the GPU from COO arrays that already live in HBM.
//
// Method: per-id rating counts with integer atomics -> strip boundaries on the host (m + n
// numbers, exact integer arithmetic shared with the host partitioner) -> one 64-bit key per
// rating, (block id L, row inside its strip, column inside its strip) from the most to the
// least significant bits, payload = original position -> stable least-significant-digit radix
// sort over the used bits, 8 bits per pass -> keys decoded into the packed row / column
// arrays, values gathered through the payload (which stays on the device as the permutation).  The payload starts in ascending original
// position and every pass is stable, so equal (L, row, column) stay in original order: the
// result is the order (L, row, column, original position) the host partitioner produces.
#include "mf_internal.h"

#include <algorithm>
#include <cstdlib>

#include "../../include/mf_sgd.h"

namespace mf {
namespace {

constexpr int kSortThreads = 256;
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kSortItems = 16;                           // keys per thread
constexpr int kSortTile = kSortThreads * kSortItems;     // keys per workgroup and pass
constexpr int kWaveSpan = kWave * kSortItems;            // consecutive keys owned by one wavefront
constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
static_assert(kRadix == kSortThreads, "one thread per digit value in the tile-level scans");
constexpr int kScanChunk = kSortThreads * 16;

struct DeviceBuffer {
    void* p = nullptr;
    ~DeviceBuffer() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, std::max<size_t>(bytes, 256)); }
    template <class T> T* as() const { return (T*)p; }
};

// ------------------------------------------------------------------------------------ kernels
__global__ __launch_bounds__(kSortThreads) void count_degrees(
    const int32_t* __restrict__ rows, const int32_t* __restrict__ cols, int64_t nnz, int32_t m, int32_t n,
    int32_t* __restrict__ row_degree, int32_t* __restrict__ col_degree, int32_t* __restrict__ bad)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < nnz; t += stride) {
        const int32_t u = rows[t], v = cols[t];
        if (u < 0 || u >= m || v < 0 || v >= n) {
            *bad = 1;
            continue;
        }
        if (row_degree) atomicAdd(&row_degree[u], 1);
        if (col_degree) atomicAdd(&col_degree[v], 1);
    }
}

// Rating counts of an axis short enough for a private histogram per workgroup in LDS (the ids of
// a skewed axis repeat often: LDS atomics instead of contended ones in the L2); the private counts
// are added to the global ones at the end.  Dynamic LDS: size * 4 bytes.
__global__ __launch_bounds__(1024) void count_ids_lds(const int32_t* __restrict__ ids, int64_t nnz, int32_t size,
                                                     int32_t* __restrict__ degree)
{
    extern __shared__ int32_t priv[];
    for (int i = threadIdx.x; i < size; i += blockDim.x) priv[i] = 0;
    __syncthreads();
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < nnz; t += stride) {
        const int32_t x = ids[t];
        if (x >= 0 && x < size) atomicAdd(&priv[x], 1);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < size; i += blockDim.x)
        if (priv[i] != 0) atomicAdd(&degree[i], priv[i]);
}

// key = L << (ubits + vbits) | (u - first row of its strip) << vbits | (v - first column of its strip)
__global__ __launch_bounds__(kSortThreads) void make_keys(
    const int32_t* __restrict__ rows, const int32_t* __restrict__ cols, int64_t nnz,
    const int32_t* __restrict__ row_strip, const int32_t* __restrict__ col_strip,
    const int32_t* __restrict__ row_bounds, const int32_t* __restrict__ col_bounds, int32_t gr, int32_t gc,
    int ubits, int vbits, const uint32_t* __restrict__ row_shift, uint64_t* __restrict__ keys,
    uint32_t* __restrict__ payload)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < nnz; t += stride) {
        const int32_t u = rows[t], v = cols[t];
        const int32_t a = row_strip[u], b = col_strip[v];
        int32_t s = b - a;
        if (s < 0) s += gc;
        const int64_t L = (int64_t)s * gr + a;
        uint64_t ur = (uint64_t)(u - row_bounds[a]);
        // seeded row order: the key holds the row's place in its strip instead of its offset
        if (row_shift) ur = row_order_rank((uint32_t)ur, row_shift[a], (uint32_t)(row_bounds[a + 1] - row_bounds[a]));
        const uint64_t vr = (uint64_t)(v - col_bounds[b]);
        keys[t] = ((uint64_t)L << (ubits + vbits)) | (ur << vbits) | vr;
        payload[t] = (uint32_t)t;
    }
}

// First packed position of every block, read off the sorted keys: position i starts block L_i and
// every empty block between L_(i-1) and L_i; the last thread closes the table.
__global__ __launch_bounds__(kSortThreads) void block_starts(const uint64_t* __restrict__ keys, int64_t nnz, int shift,
                                                           int64_t nblocks, uint32_t* __restrict__ block_ptr)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nnz; i += stride) {
        const int64_t L = (int64_t)(keys[i] >> shift);
        const int64_t before = i > 0 ? (int64_t)(keys[i - 1] >> shift) : -1;
        for (int64_t x = before + 1; x <= L; ++x) block_ptr[x] = (uint32_t)i;
        if (i == nnz - 1)
            for (int64_t x = L + 1; x <= nblocks; ++x) block_ptr[x] = (uint32_t)nnz;
    }
}

__device__ __forceinline__ int digit_of(uint64_t key, int shift) { return (int)((key >> shift) & (kRadix - 1)); }

// Exclusive prefix sum of one value per thread over the workgroup (kSortThreads threads).
__device__ __forceinline__ uint32_t group_exclusive_scan(uint32_t x, uint32_t* tmp /* kSortThreads */, uint32_t* total)
{
    const int tid = threadIdx.x;
    tmp[tid] = x;
    __syncthreads();
    for (int d = 1; d < kSortThreads; d <<= 1) {
        uint32_t add = tid >= d ? tmp[tid - d] : 0u;
        __syncthreads();
        tmp[tid] += add;
        __syncthreads();
    }
    const uint32_t incl = tmp[tid];
    if (total) *total = tmp[kSortThreads - 1];
    __syncthreads();
    return incl - x;
}

// Digit histogram of one tile; tile_hist is [digit][tile] so that its exclusive prefix sum is
// the first output position of (digit, tile) in the stable order.
__global__ __launch_bounds__(kSortThreads) void radix_histogram(
    const uint64_t* __restrict__ keys, int64_t count, int shift, uint32_t* __restrict__ tile_hist, int64_t ntiles)
{
    __shared__ uint32_t hist[kRadix];
    hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        const int64_t i = base + r * kSortThreads + threadIdx.x;
        if (i < count) atomicAdd(&hist[digit_of(keys[i], shift)], 1u);
    }
    __syncthreads();
    tile_hist[(int64_t)threadIdx.x * ntiles + blockIdx.x] = hist[threadIdx.x];
}

// Exclusive prefix sum over `count` 32-bit values in three steps: sums of chunks, prefix of the
// chunk sums (one workgroup), prefix inside every chunk plus its chunk's offset.
__global__ __launch_bounds__(kSortThreads) void scan_chunk_sums(const uint32_t* __restrict__ x, int64_t count,
                                                              uint32_t* __restrict__ sums)
{
    __shared__ uint32_t tmp[kSortThreads];
    const int64_t base = (int64_t)blockIdx.x * kScanChunk;
    uint32_t s = 0;
    for (int j = threadIdx.x; j < kScanChunk; j += kSortThreads)
        if (base + j < count) s += x[base + j];
    uint32_t total;
    group_exclusive_scan(s, tmp, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kSortThreads) void scan_of_sums(uint32_t* __restrict__ sums, int64_t nchunks)
{
    __shared__ uint32_t tmp[kSortThreads];
    const int64_t per = (nchunks + kSortThreads - 1) / kSortThreads;
    const int64_t b = std::min<int64_t>(nchunks, per * threadIdx.x), e = std::min<int64_t>(nchunks, b + per);
    uint32_t s = 0;
    for (int64_t i = b; i < e; ++i) s += sums[i];
    uint32_t run = group_exclusive_scan(s, tmp, nullptr);
    for (int64_t i = b; i < e; ++i) {
        const uint32_t v = sums[i];
        sums[i] = run;
        run += v;
    }
}

__global__ __launch_bounds__(kSortThreads) void scan_apply(uint32_t* __restrict__ x, int64_t count,
                                                         const uint32_t* __restrict__ sums)
{
    __shared__ uint32_t tmp[kSortThreads];
    constexpr int kPer = kScanChunk / kSortThreads;
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kPer;
    uint32_t v[kPer];
    uint32_t s = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        v[j] = base + j < count ? x[base + j] : 0u;
        s += v[j];
    }
    uint32_t run = group_exclusive_scan(s, tmp, nullptr) + sums[blockIdx.x];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        if (base + j < count) x[base + j] = run;
        run += v[j];
    }
}

// One stable pass.  Wavefront w of the workgroup owns the consecutive keys
// [tile*kSortTile + w*kWaveSpan, +kWaveSpan) and reads them 64 at a time in order, so "earlier
// in the input" means (wavefront, round, lane) in lexicographic order.  For every key the rank
// among the earlier keys of the tile with the same digit is: keys of earlier wavefronts (from
// the per-wavefront totals) + earlier rounds of this wavefront (a running count per digit, kept
// by the wavefront in LDS) + lower lanes of this round (from eight ballots).  The tile is then
// reordered through LDS, so that the global writes of one digit are consecutive.
__global__ __launch_bounds__(kSortThreads) void radix_scatter(
    const uint64_t* __restrict__ keys_in, const uint32_t* __restrict__ payload_in, uint64_t* __restrict__ keys_out,
    uint32_t* __restrict__ payload_out, int64_t count, int shift, const uint32_t* __restrict__ tile_first,
    int64_t ntiles)
{
    __shared__ uint32_t wave_count[kSortWaves][kRadix];
    __shared__ uint32_t digit_start[kRadix];    // first tile-local position of every digit
    __shared__ uint32_t global_first[kRadix];   // first output position of (digit, this tile)
    __shared__ uint32_t tmp[kSortThreads];
    __shared__ uint64_t tile_keys[kSortTile];
    __shared__ uint32_t tile_payload[kSortTile];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    for (int w = 0; w < kSortWaves; ++w) wave_count[w][tid] = 0;
    global_first[tid] = tile_first[(int64_t)tid * ntiles + blockIdx.x];
    __syncthreads();

    const int64_t tile_base = (int64_t)blockIdx.x * kSortTile;
    const int64_t wave_base = tile_base + (int64_t)wave * kWaveSpan;
    uint64_t key[kSortItems];
    uint32_t pay[kSortItems];
    uint32_t rank[kSortItems];
    volatile uint32_t* mine = wave_count[wave];
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        const int64_t i = wave_base + r * kWave + lane;
        const bool valid = i < count;
        key[r] = valid ? keys_in[i] : 0;
        pay[r] = valid ? payload_in[i] : 0;
    }
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        const bool valid = wave_base + r * kWave + lane < count;
        const int d = digit_of(key[r], shift);
        // lanes of this round that hold a valid key with the same digit
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < kRadixBits; ++bit) {
            const bool one = (d >> bit) & 1;
            const uint64_t with_one = __ballot(one);
            peers &= one ? with_one : ~with_one;
        }
        const uint32_t lower = (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
        const uint32_t before = mine[d];          // every lane of `peers` reads the same counter ...
        rank[r] = before + lower;
        if (valid && lower == 0) mine[d] = before + (uint32_t)__popcll(peers);   // ... then its first lane advances it
    }
    __syncthreads();
    {   // thread = digit: totals of the earlier wavefronts, and of the tile
        uint32_t run = 0;
        for (int w = 0; w < kSortWaves; ++w) {
            const uint32_t c = wave_count[w][tid];
            wave_count[w][tid] = run;
            run += c;
        }
        digit_start[tid] = group_exclusive_scan(run, tmp, nullptr);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        if (wave_base + r * kWave + lane < count) {
            const int d = digit_of(key[r], shift);
            const uint32_t pos = digit_start[d] + wave_count[wave][d] + rank[r];
            if (pos < (uint32_t)kSortTile) {   // always true; keeps a wrong count from leaving the arrays
                tile_keys[pos] = key[r];
                tile_payload[pos] = pay[r];
            }
        }
    }
    __syncthreads();
    const int in_tile = (int)std::min<int64_t>(kSortTile, count - tile_base);
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        const int j = r * kSortThreads + tid;
        if (j < in_tile) {
            const uint64_t k = tile_keys[j];
            const int d = digit_of(k, shift);
            const int64_t dest = (int64_t)global_first[d] + (j - (int)digit_start[d]);
            if (dest >= 0 && dest < count) {   // always true, see above
                keys_out[dest] = k;
                payload_out[dest] = tile_payload[j];
            }
        }
    }
}

__global__ __launch_bounds__(kSortThreads) void unpack_keys(
    const uint64_t* __restrict__ keys, const uint32_t* __restrict__ payload, int64_t nnz,
    const int32_t* __restrict__ row_bounds, const int32_t* __restrict__ col_bounds, int32_t gr, int32_t gc,
    int ubits, int vbits, const uint32_t* __restrict__ row_shift, const uint32_t* __restrict__ row_inverse,
    const float* __restrict__ vals, int32_t* __restrict__ U, int32_t* __restrict__ V, float* __restrict__ R,
    uint32_t* __restrict__ perm)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nnz; i += stride) {
        const uint64_t k = keys[i];
        const int64_t L = (int64_t)(k >> (ubits + vbits));
        const int32_t a = (int32_t)(L % gr), s = (int32_t)(L / gr);
        int32_t b = a + s;
        if (b >= gc) b -= gc;
        uint64_t ur = (k >> vbits) & ((1ull << ubits) - 1ull);
        if (row_shift) {
            // undo the affine map: offset = (place - shift) * prime^-1 mod width
            const uint64_t width = (uint64_t)(row_bounds[a + 1] - row_bounds[a]);
            ur = ((ur + width - row_shift[a]) % width) * row_inverse[a] % width;
        }
        U[i] = row_bounds[a] + (int32_t)ur;
        V[i] = col_bounds[b] + (int32_t)(k & ((1ull << vbits) - 1ull));
        const uint32_t t = payload[i];
        R[i] = vals[t];
        perm[i] = t;
    }
}

// Word w of `words`: bit j set when packed rating 64*w + j has another row index than the
// rating before it (rating 0 always).  One wavefront per word.
__global__ __launch_bounds__(kSortThreads) void row_start_words(const int32_t* __restrict__ U, int64_t nnz,
                                                              uint64_t* __restrict__ words, int64_t nwords)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t waves = (int64_t)gridDim.x * kSortWaves;
    for (int64_t w = (int64_t)blockIdx.x * kSortWaves + (threadIdx.x >> 6); w < nwords; w += waves) {
        const int64_t i = w * kWave + lane;
        const bool start = i < nnz && (i == 0 || U[i] != U[i - 1]);
        const uint64_t word = __ballot(start);
        if (lane == 0) words[w] = word;
    }
}

int bits_for(int64_t values)   // bits needed to tell `values` different numbers apart
{
    int b = 0;
    while (((int64_t)1 << b) < values) ++b;
    return b;
}

int streaming_groups(int64_t items) { return (int)std::max<int64_t>(1, std::min<int64_t>((items + kSortThreads - 1) / kSortThreads, 256 * 16)); }

}  // namespace

#define PD_HIP(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            err = std::string(#call) + ": " + hipGetErrorString(e_);                   \
            return e_ == hipErrorOutOfMemory ? MF_ENOMEM : MF_EDEVICE;                 \
        }                                                                              \
    } while (0)

int build_partition_device(const int32_t* d_rows, const int32_t* d_cols, const float* d_vals, int64_t nnz,
                           int64_t m, int64_t n, int32_t gr, int32_t gc, int32_t split, uint64_t row_seed,
                           int32_t* dU, int32_t* dV, float* dR, uint32_t* d_perm, Partition& out, RowStarts& rs,
                           hipStream_t stream, std::string& err)
{
    const int64_t nblocks = (int64_t)gr * gc;
    const bool balanced = split != MF_SPLIT_EQUAL_WIDTH;
    out.nnz = nnz;
    out.gr = gr;
    out.gc = gc;

    // ---- range check and rating counts per row and per column
    DeviceBuffer row_degree, col_degree, flag;
    PD_HIP(flag.alloc(4));
    PD_HIP(hipMemsetAsync(flag.p, 0, 4, stream));
    if (balanced) {
        PD_HIP(row_degree.alloc((size_t)m * 4));
        PD_HIP(col_degree.alloc((size_t)n * 4));
        PD_HIP(hipMemsetAsync(row_degree.p, 0, (size_t)m * 4, stream));
        PD_HIP(hipMemsetAsync(col_degree.p, 0, (size_t)n * 4, stream));
    }
    if (nnz > 0) {
        // an axis whose counters fit the LDS is counted there, the other one (and the range check) with
        // global atomics
        constexpr int64_t kLdsCounters = 36 * 1024;
        const bool rows_in_lds = balanced && m <= kLdsCounters, cols_in_lds = balanced && n <= kLdsCounters;
        hipLaunchKernelGGL(count_degrees, dim3(streaming_groups(nnz)), dim3(kSortThreads), 0, stream, d_rows, d_cols,
                           nnz, (int32_t)m, (int32_t)n, rows_in_lds ? nullptr : row_degree.as<int32_t>(),
                           cols_in_lds ? nullptr : col_degree.as<int32_t>(), flag.as<int32_t>());
        PD_HIP(hipGetLastError());
        static bool raised[64] = {};
        int dev = 0;
        PD_HIP(hipGetDevice(&dev));
        if ((rows_in_lds || cols_in_lds) && dev >= 0 && dev < 64 && !raised[dev]) {
            PD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&count_ids_lds),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kLdsCounters * 4)));
            raised[dev] = true;
        }
        const int groups = (int)std::max<int64_t>(1, std::min<int64_t>((nnz + 16383) / 16384, 512));
        if (rows_in_lds) {
            hipLaunchKernelGGL(count_ids_lds, dim3(groups), dim3(1024), (size_t)m * 4, stream, d_rows, nnz, (int32_t)m,
                               row_degree.as<int32_t>());
            PD_HIP(hipGetLastError());
        }
        if (cols_in_lds) {
            hipLaunchKernelGGL(count_ids_lds, dim3(groups), dim3(1024), (size_t)n * 4, stream, d_cols, nnz, (int32_t)n,
                               col_degree.as<int32_t>());
            PD_HIP(hipGetLastError());
        }
    }
    int32_t bad = 0;
    PD_HIP(hipMemcpyAsync(&bad, flag.p, 4, hipMemcpyDeviceToHost, stream));
    PD_HIP(hipStreamSynchronize(stream));
    if (bad) {
        err = "a row or column index lies outside the matrix";
        return MF_ERANGE;
    }
    if (balanced) {
        std::vector<int32_t> deg((size_t)std::max(m, n));
        const bool width_weight = split == MF_SPLIT_NNZ_WIDTH_BALANCED;
        PD_HIP(hipMemcpy(deg.data(), row_degree.p, (size_t)m * 4, hipMemcpyDeviceToHost));
        bounds_from_degrees(deg.data(), nnz, m, gr, width_weight, out.row_bounds);
        PD_HIP(hipMemcpy(deg.data(), col_degree.p, (size_t)n * 4, hipMemcpyDeviceToHost));
        bounds_from_degrees(deg.data(), nnz, n, gc, width_weight, out.col_bounds);
    } else {
        equal_width_bounds(m, gr, out.row_bounds);
        equal_width_bounds(n, gc, out.col_bounds);
    }
    out.block_ptr.assign((size_t)nblocks + 1, 0);
    out.perm.clear();
    rs.bits.clear();
    if (nnz == 0) return MF_OK;

    // ---- key layout
    int32_t widest_row = 1, widest_col = 1;
    for (int32_t a = 0; a < gr; ++a) widest_row = std::max(widest_row, out.row_bounds[a + 1] - out.row_bounds[a]);
    for (int32_t b = 0; b < gc; ++b) widest_col = std::max(widest_col, out.col_bounds[b + 1] - out.col_bounds[b]);
    const int ubits = bits_for(widest_row), vbits = bits_for(widest_col), lbits = bits_for(nblocks);
    const int key_bits = ubits + vbits + lbits;
    if (key_bits > 64) {
        err = "grid and strip widths need more than 64 key bits on the device; use mf_load_blocks";
        return MF_EINVAL;
    }

    // ---- strip lookup tables and boundaries on the device (the degree buffers are reused)
    std::vector<int32_t> table;
    DeviceBuffer row_strip, col_strip, d_row_bounds, d_col_bounds, block_count;
    PD_HIP(row_strip.alloc((size_t)m * 4));
    PD_HIP(col_strip.alloc((size_t)n * 4));
    PD_HIP(d_row_bounds.alloc(((size_t)gr + 1) * 4));
    PD_HIP(d_col_bounds.alloc(((size_t)gc + 1) * 4));
    PD_HIP(block_count.alloc(((size_t)nblocks + 1) * 4));   // first packed position of every block
    strip_table(out.row_bounds, m, table);
    PD_HIP(hipMemcpy(row_strip.p, table.data(), (size_t)m * 4, hipMemcpyHostToDevice));
    strip_table(out.col_bounds, n, table);
    PD_HIP(hipMemcpy(col_strip.p, table.data(), (size_t)n * 4, hipMemcpyHostToDevice));
    PD_HIP(hipMemcpy(d_row_bounds.p, out.row_bounds.data(), ((size_t)gr + 1) * 4, hipMemcpyHostToDevice));
    PD_HIP(hipMemcpy(d_col_bounds.p, out.col_bounds.data(), ((size_t)gc + 1) * 4, hipMemcpyHostToDevice));
    // seeded row order: per row strip the shift of the affine map and the inverse of its multiplier
    DeviceBuffer d_row_shift, d_row_inverse;
    if (row_seed) {
        std::vector<uint32_t> shift((size_t)gr), inverse((size_t)gr);
        for (int32_t a = 0; a < gr; ++a) {
            const int64_t width = std::max(1, out.row_bounds[a + 1] - out.row_bounds[a]);
            shift[(size_t)a] = row_order_shift(row_seed, a, (int32_t)width);
            // inverse of the prime modulo width by the extended Euclidean algorithm
            int64_t r0 = width, r1 = (int64_t)(kRowOrderPrime % (uint64_t)width), t0 = 0, t1 = 1;
            while (r1 != 0) {
                const int64_t q = r0 / r1;
                const int64_t r2 = r0 - q * r1, t2 = t0 - q * t1;
                r0 = r1; r1 = r2; t0 = t1; t1 = t2;
            }
            inverse[(size_t)a] = (uint32_t)(((t0 % width) + width) % width);   // width 1: 0, the only offset
        }
        PD_HIP(d_row_shift.alloc((size_t)gr * 4));
        PD_HIP(d_row_inverse.alloc((size_t)gr * 4));
        PD_HIP(hipMemcpy(d_row_shift.p, shift.data(), (size_t)gr * 4, hipMemcpyHostToDevice));
        PD_HIP(hipMemcpy(d_row_inverse.p, inverse.data(), (size_t)gr * 4, hipMemcpyHostToDevice));
    }

    // ---- keys, payload, block sizes
    const int64_t ntiles = (nnz + kSortTile - 1) / kSortTile;
    const int64_t hist_len = (int64_t)kRadix * ntiles;
    const int64_t nchunks = (hist_len + kScanChunk - 1) / kScanChunk;
    DeviceBuffer keys[2], payload[2], tile_hist, chunk_sums;
    for (int i = 0; i < 2; ++i) {
        PD_HIP(keys[i].alloc((size_t)nnz * 8));
        PD_HIP(payload[i].alloc((size_t)nnz * 4));
    }
    PD_HIP(tile_hist.alloc((size_t)hist_len * 4));
    PD_HIP(chunk_sums.alloc((size_t)nchunks * 4));
    hipLaunchKernelGGL(make_keys, dim3(streaming_groups(nnz)), dim3(kSortThreads), 0, stream, d_rows, d_cols, nnz,
                       row_strip.as<int32_t>(), col_strip.as<int32_t>(), d_row_bounds.as<int32_t>(),
                       d_col_bounds.as<int32_t>(), gr, gc, ubits, vbits, row_seed ? d_row_shift.as<uint32_t>() : nullptr,
                       keys[0].as<uint64_t>(), payload[0].as<uint32_t>());
    PD_HIP(hipGetLastError());

    // ---- stable radix passes over the used bits
    int cur = 0;
    for (int shift = 0; shift < key_bits; shift += kRadixBits) {
        hipLaunchKernelGGL(radix_histogram, dim3((unsigned)ntiles), dim3(kSortThreads), 0, stream,
                           keys[cur].as<uint64_t>(), nnz, shift, tile_hist.as<uint32_t>(), ntiles);
        hipLaunchKernelGGL(scan_chunk_sums, dim3((unsigned)nchunks), dim3(kSortThreads), 0, stream,
                           tile_hist.as<uint32_t>(), hist_len, chunk_sums.as<uint32_t>());
        hipLaunchKernelGGL(scan_of_sums, dim3(1), dim3(kSortThreads), 0, stream, chunk_sums.as<uint32_t>(), nchunks);
        hipLaunchKernelGGL(scan_apply, dim3((unsigned)nchunks), dim3(kSortThreads), 0, stream,
                           tile_hist.as<uint32_t>(), hist_len, chunk_sums.as<uint32_t>());
        hipLaunchKernelGGL(radix_scatter, dim3((unsigned)ntiles), dim3(kSortThreads), 0, stream,
                           keys[cur].as<uint64_t>(), payload[cur].as<uint32_t>(), keys[cur ^ 1].as<uint64_t>(),
                           payload[cur ^ 1].as<uint32_t>(), nnz, shift, tile_hist.as<uint32_t>(), ntiles);
        PD_HIP(hipGetLastError());
        cur ^= 1;
    }

    // ---- packed arrays
    hipLaunchKernelGGL(unpack_keys, dim3(streaming_groups(nnz)), dim3(kSortThreads), 0, stream,
                       keys[cur].as<uint64_t>(), payload[cur].as<uint32_t>(), nnz, d_row_bounds.as<int32_t>(),
                       d_col_bounds.as<int32_t>(), gr, gc, ubits, vbits,
                       row_seed ? d_row_shift.as<uint32_t>() : nullptr,
                       row_seed ? d_row_inverse.as<uint32_t>() : nullptr, d_vals, dU, dV, dR, d_perm);
    PD_HIP(hipGetLastError());
    hipLaunchKernelGGL(block_starts, dim3(streaming_groups(nnz)), dim3(kSortThreads), 0, stream,
                       keys[cur].as<uint64_t>(), nnz, ubits + vbits, nblocks, block_count.as<uint32_t>());
    PD_HIP(hipGetLastError());
    const int64_t nwords = (nnz + kWave - 1) / kWave;
    DeviceBuffer words;
    PD_HIP(words.alloc((size_t)nwords * 8));
    hipLaunchKernelGGL(row_start_words, dim3(streaming_groups(nwords * kWave / kSortWaves)), dim3(kSortThreads), 0, stream,
                       dU, nnz, words.as<uint64_t>(), nwords);
    PD_HIP(hipGetLastError());
    PD_HIP(hipStreamSynchronize(stream));

    // ---- what the host needs for the work lists: block boundaries and where the row runs begin
    {
        std::vector<uint32_t> starts((size_t)nblocks + 1);
        PD_HIP(hipMemcpy(starts.data(), block_count.p, ((size_t)nblocks + 1) * 4, hipMemcpyDeviceToHost));
        for (int64_t L = 0; L <= nblocks; ++L) out.block_ptr[(size_t)L] = (int64_t)starts[(size_t)L];
    }
    rs.bits.resize((size_t)nwords);
    PD_HIP(hipMemcpy(rs.bits.data(), words.p, (size_t)nwords * 8, hipMemcpyDeviceToHost));
    return MF_OK;
}

}  // namespace mf
