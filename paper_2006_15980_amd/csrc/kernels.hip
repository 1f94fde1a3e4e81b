// Device code of libmf_sgd for gfx950 (CDNA4, 64-wide wavefronts).
//
// All SGD kernels run the training step of the paper's Algorithm 1 -- e = r - p.q, then
// p += lr*(e*q - lambda*p), q += lr*(e*p - lambda*q) with the old p on the right -- one rating at
// a time per wavefront, the k factors of a row spread over the lanes, the dot product reduced with
// DPP cross-lane adds.
//   sgd_chunks    : one wavefront per work-list entry, rows of P and Qt in global memory
//                   (deterministic mode on any grid; Hogwild fallback with L2 atomics).
//   sgd_block_lds : one workgroup per block of a stratum; the block's strip of Qt lives in LDS
//                   (fp32 for the deterministic mode, 32-bit fixed point + integer atomics for
//                   Hogwild), rows of P stream through registers; in Hogwild mode the few rows
//                   of P that are shared out over several wavefronts sit in LDS beside the strip,
//                   and the strip may be packed: only the columns in which the block has a rating.
//   sgd_ring_lds  : the same block body, one launch per epoch: workgroup a keeps block row a and
//                   the column strips are handed from workgroup to workgroup with bounded waits.
//   rmse_partial / rmse_final : sum of squared prediction errors (Eq. 1 against the rating),
//                   double precision, fixed reduction order.
//   init_fill     : counter-based uniform initial factors.
//   mark_touched  : per block, the columns of its strip in which it has a rating (for packing).
//
// This is a gather / dot / scatter over rows of 128..1024 bytes with about half a flop per byte:
// there is no MFMA here; the lanes hold rows in registers, consecutive ratings of one matrix row
// reuse p_u from registers, and the rows of later ratings are requested ahead of their use.
#include <algorithm>
#include <utility>

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "../../include/mf_sgd.h"
#include "mf_internal.h"

namespace mf {
namespace {

// ---------------------------------------------------------------------------------- row access
// A factor row of K elements is spread over the lanes of a wavefront, VEC values per lane:
//   fp32     : value j of lane l is element l + 64*j, so every load / store / atomic instruction
//              of the wavefront covers 256 contiguous bytes; lanes >= K are idle (K = 32);
//   binary16 : values 2j, 2j+1 of lane l are the element pair 2*l + 128*j, +1 (one 32-bit word,
//              which is what the packed binary16 atomic add needs); lanes >= K/2 are idle.
// Idle lanes hold zeros and never touch memory.
template <typename T, int K>
struct RowShape;
template <int K>
struct RowShape<float, K> {
    static constexpr int VEC = K >= 64 ? K / 64 : 1;
    static constexpr int ACTIVE = K >= 64 ? 64 : K;
};
template <int K>
struct RowShape<__half, K> {
    static constexpr int VEC = K >= 128 ? K / 64 : 2;
    static constexpr int ACTIVE = K >= 128 ? 64 : K / 2;
};

template <int VEC>
struct Row {
    float x[VEC];
};

// 32-bit load; FRESH = read through to the die's L2 (agent-scope atomic load) instead of the
// compute unit's private L1, which atomic updates made by other compute units do not refresh.
template <bool FRESH>
__device__ __forceinline__ unsigned load_word(const unsigned* p)
{
    if constexpr (FRESH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}

__device__ __forceinline__ float2 unpack_half2(unsigned w)
{
    __half2 h = *reinterpret_cast<__half2*>(&w);
    return make_float2(__low2float(h), __high2float(h));
}

__device__ __forceinline__ unsigned pack_half2(float a, float b)
{
    __half2 h = __floats2half2_rn(a, b);
    return *reinterpret_cast<unsigned*>(&h);
}

template <int VEC, bool FRESH>
__device__ __forceinline__ Row<VEC> load_row(const float* row_ptr, int lane, bool active)
{
    Row<VEC> r;
#pragma unroll
    for (int j = 0; j < VEC; ++j) r.x[j] = 0.f;
    if (active) {
#pragma unroll
        for (int j = 0; j < VEC; ++j)
            r.x[j] = __uint_as_float(load_word<FRESH>(reinterpret_cast<const unsigned*>(row_ptr) + lane + kWave * j));
    }
    return r;
}

template <int VEC, bool FRESH>
__device__ __forceinline__ Row<VEC> load_row(const __half* row_ptr, int lane, bool active)
{
    Row<VEC> r;
#pragma unroll
    for (int j = 0; j < VEC; ++j) r.x[j] = 0.f;
    if (active) {
#pragma unroll
        for (int j = 0; j < VEC / 2; ++j) {
            float2 t = unpack_half2(load_word<FRESH>(reinterpret_cast<const unsigned*>(row_ptr) + lane + kWave * j));
            r.x[2 * j] = t.x;
            r.x[2 * j + 1] = t.y;
        }
    }
    return r;
}

template <int VEC>
__device__ __forceinline__ void store_row(float* row_ptr, int lane, bool active, const Row<VEC>& r)
{
    if (!active) return;
#pragma unroll
    for (int j = 0; j < VEC; ++j) row_ptr[lane + kWave * j] = r.x[j];
}

// binary16 storage: the row kept in registers already holds values on the binary16 grid
// (see quantise), so the conversion below is exact.
template <int VEC>
__device__ __forceinline__ void store_row(__half* row_ptr, int lane, bool active, const Row<VEC>& r)
{
    if (!active) return;
#pragma unroll
    for (int j = 0; j < VEC / 2; ++j)
        reinterpret_cast<unsigned*>(row_ptr)[lane + kWave * j] = pack_half2(r.x[2 * j], r.x[2 * j + 1]);
}

// A row as it lies in memory, requested now and turned into values only where it is used: the
// registers of a row on its way hold the loaded words (binary16: half as many as values), and
// the conversion cannot drift up to the load, where it would wait for the data at once.
template <typename T, int K>
struct StoredRow {
    static constexpr int WORDS = RowShape<T, K>::VEC * (int)sizeof(T) / 4;
    unsigned w[WORDS];
};

template <typename T, int K, bool FRESH>
__device__ __forceinline__ StoredRow<T, K> request_row(const T* row_ptr, int lane, bool active)
{
    StoredRow<T, K> r;
#pragma unroll
    for (int j = 0; j < StoredRow<T, K>::WORDS; ++j)
        r.w[j] = active ? load_word<FRESH>(reinterpret_cast<const unsigned*>(row_ptr) + lane + kWave * j) : 0u;
    return r;
}

template <typename T, int K>
__device__ __forceinline__ Row<RowShape<T, K>::VEC> row_values(const StoredRow<T, K>& r)
{
    Row<RowShape<T, K>::VEC> out;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int j = 0; j < StoredRow<T, K>::WORDS; ++j) {
            const float2 t = unpack_half2(r.w[j]);
            out.x[2 * j] = t.x;
            out.x[2 * j + 1] = t.y;
        }
    } else {
#pragma unroll
        for (int j = 0; j < StoredRow<T, K>::WORDS; ++j) out.x[j] = __uint_as_float(r.w[j]);
    }
    return out;
}

// row += d with hardware floating-point atomic adds executed in the L2 (no value returned).
template <int VEC>
__device__ __forceinline__ void atomic_add_row(float* row_ptr, int lane, bool active, const Row<VEC>& d)
{
    if (!active) return;
#pragma unroll
    for (int j = 0; j < VEC; ++j) unsafeAtomicAdd(row_ptr + lane + kWave * j, d.x[j]);
}

template <int VEC>
__device__ __forceinline__ void atomic_add_row(__half* row_ptr, int lane, bool active, const Row<VEC>& d)
{
    if (!active) return;
#pragma unroll
    for (int j = 0; j < VEC / 2; ++j)
        unsafeAtomicAdd(reinterpret_cast<__half2*>(row_ptr) + lane + kWave * j,
                        __floats2half2_rn(d.x[2 * j], d.x[2 * j + 1]));
}

// Values leave a step on the grid of the storage type: fp32 as they are, binary16 rounded to
// nearest even after EVERY step, also while a row stays in registers across several ratings.
// The conversion takes a finished fp32 value: the empty asm keeps the compiler from folding the
// producing multiply-add into a mixed-precision instruction that would round only once.
__device__ __forceinline__ __half round_to_half(float x)
{
    asm("" : "+v"(x));
    return __float2half_rn(x);
}

template <typename T>
__device__ __forceinline__ float quantise(float x)
{
    if constexpr (sizeof(T) == 2) return __half2float(round_to_half(x));
    return x;
}

// ------------------------------------------------------------------------------ wave reduction
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float x)
{
    int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
    return x + __int_as_float(moved);
}

// Sum over the 64 lanes, returned as a wave-uniform value.  Steps: neighbours inside a quad,
// quad pairs, mirrored halves of 8, mirrored row of 16, then lane 15 of each row into the next
// row (rows 1 and 3), then lane 31 into rows 2 and 3; lane 63 ends up with the total.
__device__ __forceinline__ float wave_sum(float x)
{
    x = dpp_add<0xB1, 0xf>(x);    // quad_perm [1,0,3,2]
    x = dpp_add<0x4E, 0xf>(x);    // quad_perm [2,3,0,1]
    x = dpp_add<0x141, 0xf>(x);   // row_half_mirror
    x = dpp_add<0x140, 0xf>(x);   // row_mirror
    x = dpp_add<0x142, 0xa>(x);   // row_bcast15 into rows 1 and 3
    x = dpp_add<0x143, 0xc>(x);   // row_bcast31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// The same reduction on doubles (each step moves the two 32-bit halves).  Used where the sum
// must not depend on rounding order: the deterministic mode with binary16 storage.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_add_f64(double x)
{
    const long long bits = __double_as_longlong(x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)bits, CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(bits >> 32), CTRL, ROW_MASK, 0xf, false);
    return x + __longlong_as_double(((long long)hi << 32) | (unsigned)lo);
}

__device__ __forceinline__ double wave_sum_f64_dpp(double x)
{
    x = dpp_add_f64<0xB1, 0xf>(x);
    x = dpp_add_f64<0x4E, 0xf>(x);
    x = dpp_add_f64<0x141, 0xf>(x);
    x = dpp_add_f64<0x140, 0xf>(x);
    x = dpp_add_f64<0x142, 0xa>(x);
    x = dpp_add_f64<0x143, 0xc>(x);
    const long long bits = __double_as_longlong(x);
    const int lo = __builtin_amdgcn_readlane((int)bits, 63);
    const int hi = __builtin_amdgcn_readlane((int)(bits >> 32), 63);
    return __longlong_as_double(((long long)hi << 32) | (unsigned)lo);
}

__device__ __forceinline__ int uniform_lane(int v, int lane)
{
    return __builtin_amdgcn_readlane(v, lane);
}

// ------------------------------------------------------------------------------------ SGD step
// One work-list entry = `len` consecutive ratings of the packed (block-major, row-major) order.
// Invariants of the loop below, for the rating at position i of the current batch of 64:
//   p  holds row u_i of P as the sequential order would see it (kept in registers while the
//      row index does not change, written back when it changes and at the end);
//   q  holds row v_i of Qt likewise: it was requested while rating i-1 was being computed, and
//      replaced by the freshly computed row when v_i == v_{i-1} (the request was issued before
//      the write of rating i-1 and would be stale).
// HOG = false (deterministic mode): the wavefront is the only one touching its rows during the
//      launch; rows are written with plain stores.
// HOG = true (Hogwild mode): other wavefronts of the same die update rows of Qt at the same
//      time, so the change of q_v is ADDED to memory with a floating-point atomic (no update is
//      lost; the value it was computed from may be slightly out of date), and rows are read
//      past the L1.  Entries whose length has the sign bit set share their row of P with other
//      entries (a very long row cut into pieces that run concurrently): they treat p_u like
//      q_v -- re-read it for every rating and add every change atomically -- because pieces
//      that each corrected a private copy of p_u over many ratings and then added those
//      corrections up would overshoot.  All other entries own their rows of P, keep p_u in
//      registers over the whole row and store it once.
constexpr int32_t kSharedRowFlag = (int32_t)0x80000000;

template <typename T, int K, bool HOG>
__global__ __launch_bounds__(kGroupThreads) void sgd_chunks(
    T* __restrict__ P, T* __restrict__ Qt, const int32_t* __restrict__ U,
    const int32_t* __restrict__ V, const float* __restrict__ R,
    const int64_t* __restrict__ entry_begin, const int32_t* __restrict__ entry_len,
    int64_t first_entry, float lr, float lambda)
{
    constexpr int VEC = RowShape<T, K>::VEC;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t entry = first_entry + (int64_t)blockIdx.x * kWavesPerGroup + wave;
    const int32_t raw_len = entry_len[entry];
    if (raw_len == 0) return;
    const bool shared_rows = HOG && raw_len < 0;
    const int32_t len = raw_len & ~kSharedRowFlag;
    const int64_t begin = entry_begin[entry];
    const bool active = lane < RowShape<T, K>::ACTIVE;
    const float shrink = lr * lambda;

    Row<VEC> p, q, p_at_load;
    int cur_u = -1;
    // write row `row` of P back: plain store, or the accumulated change as an atomic add
    auto flush_p = [&](int row, const Row<VEC>& val) {
        if (shared_rows) {
            Row<VEC> d;
#pragma unroll
            for (int j = 0; j < VEC; ++j) d.x[j] = val.x[j] - p_at_load.x[j];
            atomic_add_row<VEC>(P + (int64_t)row * K, lane, active, d);
        } else {
            store_row<VEC>(P + (int64_t)row * K, lane, active, val);
        }
    };
    for (int32_t off = 0; off < len; off += kWave) {
        const int cnt = min(kWave, len - off);
        int mu = 0, mv = 0;
        float mr = 0.f;
        if (lane < cnt) {
            mu = U[begin + off + lane];
            mv = V[begin + off + lane];
            mr = R[begin + off + lane];
        }
        int u = uniform_lane(mu, 0);
        int v = uniform_lane(mv, 0);
        if (u != cur_u) {
            if (cur_u >= 0) flush_p(cur_u, p);
            p = load_row<VEC, HOG>(P + (int64_t)u * K, lane, active);
            p_at_load = p;
            cur_u = u;
        }
        q = load_row<VEC, HOG>(Qt + (int64_t)v * K, lane, active);
        for (int i = 0; i < cnt; ++i) {
            const float r = __int_as_float(uniform_lane(__float_as_int(mr), i));
            // request the rows of the next rating of this batch before computing this one
            const bool more = i + 1 < cnt;
            int un = u, vn = v;
            Row<VEC> pn, qn;
            if (more) {
                un = uniform_lane(mu, i + 1);
                vn = uniform_lane(mv, i + 1);
                qn = load_row<VEC, HOG>(Qt + (int64_t)vn * K, lane, active);
                if (un != u || shared_rows) pn = load_row<VEC, HOG>(P + (int64_t)un * K, lane, active);
            }
            float e;
            if constexpr (!HOG && sizeof(T) == 2) {
                // deterministic mode on binary16 storage: the value that gets rounded to binary16
                // must not depend on the summation order of the dot product, so it is summed in
                // double and rounded once
                double part = 0.0;
#pragma unroll
                for (int j = 0; j < VEC; ++j) part = fma((double)p.x[j], (double)q.x[j], part);
                e = r - (float)wave_sum_f64_dpp(part);
            } else {
                float part = 0.f;
#pragma unroll
                for (int j = 0; j < VEC; ++j) part = fmaf(p.x[j], q.x[j], part);
                e = r - wave_sum(part);
            }
            const float step = lr * e;
            Row<VEC> p2, q2;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                // p + lr*(e*q - lambda*p) as p + ((lr*e)*q - (lr*lambda)*p): the small change is
                // formed first, so that only ONE rounding happens at the magnitude of the element
                // (and none with a bias, as a precomputed factor 1 - lr*lambda would have)
                p2.x[j] = quantise<T>(p.x[j] + fmaf(step, q.x[j], -shrink * p.x[j]));
            }
            if constexpr (HOG) {
                Row<VEC> dq;
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    dq.x[j] = fmaf(step, p.x[j], -shrink * q.x[j]);
                    q2.x[j] = quantise<T>(q.x[j] + dq.x[j]);
                }
                atomic_add_row<VEC>(Qt + (int64_t)v * K, lane, active, dq);
            } else {
#pragma unroll
                for (int j = 0; j < VEC; ++j)
                    q2.x[j] = quantise<T>(q.x[j] + fmaf(step, p.x[j], -shrink * q.x[j]));
                store_row<VEC>(Qt + (int64_t)v * K, lane, active, q2);
            }
            if (more) {
                if (un != u) {
                    flush_p(u, p2);
                    p = pn;
                    p_at_load = pn;
                    cur_u = un;
                } else if (shared_rows) {
                    // publish this rating's change, go on from the re-read row plus that change
                    // (the re-read was requested before the change was added)
                    Row<VEC> d;
#pragma unroll
                    for (int j = 0; j < VEC; ++j) d.x[j] = p2.x[j] - p_at_load.x[j];
                    atomic_add_row<VEC>(P + (int64_t)u * K, lane, active, d);
#pragma unroll
                    for (int j = 0; j < VEC; ++j) p.x[j] = quantise<T>(pn.x[j] + d.x[j]);
                    p_at_load = p;
                } else {
                    p = p2;
                }
                q = (vn == v) ? q2 : qn;
                u = un;
                v = vn;
            } else {
                p = p2;
            }
        }
    }
    flush_p(cur_u, p);
}

// ------------------------------------------------------------- Hogwild with the Qt strip in LDS
// One workgroup per block of the grid.  The block's strip of Qt (its ncols columns, contiguous
// rows of Qt) is copied into LDS, the wavefronts of the workgroup share out the block's entries
// (chunks of whole matrix rows) round-robin and run the step of Algorithm 1 on them
// -- p_u in registers, q_v read from LDS and changed with LDS atomic adds, so no update of q_v
// is lost although the wavefronts do not lock anything -- and the strip is written back at the
// end.  Blocks of one launch are mutually independent, so no other workgroup touches these rows
// of P or columns of Qt meanwhile.
// The strip is held as 32-bit fixed point with kFixedBits fraction bits (range +-2^(31-bits),
// step 2^-bits, i.e. the fp32 spacing of values in [0.5, 1)): the LDS executes integer atomic
// adds at the rate of plain accesses, floating-point ones some twenty times slower (measured),
// and integer sums do not depend on the order in which the wavefronts add.
// The columns of a strip are reused once per rating of the block (tens of times each), which is
// what makes the staging pay; rows of P are used by one wavefront and stream through registers.
template <typename T>
__device__ __forceinline__ int strip_elem(int lane, int j)
{
    if constexpr (sizeof(T) == 2) return 2 * lane + 2 * kWave * (j >> 1) + (j & 1);
    return lane + kWave * j;
}

// rows of P requested ahead in the Hogwild form: kShortPrefetchDepth, or the long depth of the
// storage type (a requested binary16 row takes one register per lane, an fp32 row two)
constexpr int kLdsPrefetchDepth = 8;
constexpr int kLdsPrefetchDepthHalf = 12;
constexpr int kShortPrefetchDepth = 4;
template <typename T>
constexpr int kLongPrefetchDepth = sizeof(T) == 2 ? kLdsPrefetchDepthHalf : kLdsPrefetchDepth;
// The deterministic form has a compute unit nearly to itself (one wavefront per workgroup) and
// registers to spare: 16 rows ahead measured 5 % faster than 8 on 250 M ratings, 32 slower.
constexpr int kDetPrefetchDepth = 16;

constexpr int kFixedBits = 24;
constexpr float kToFixed = (float)(1 << kFixedBits);
constexpr float kFromFixed = 1.0f / (float)(1 << kFixedBits);

__device__ __forceinline__ int to_fixed(float x)
{
    // saturating: factors anywhere near +-128 mean the training has already diverged
    return __float2int_rn(fminf(fmaxf(x * kToFixed, -2147483520.f), 2147483520.f));
}

__device__ __forceinline__ float from_fixed(int x) { return (float)x * kFromFixed; }

// Range watch of the fixed-point strip.  A strip word wraps round at +-2^31 (+-128.0).  Every add
// of a wavefront follows its own read of the same word, and at most 16 wavefronts add to a strip
// at a time, so no word can reach +-2^31 as long as every value READ stays below kWatchValue and
// every single change below kWatchChange (2^30 + 16 * 2^26 = 2^31); the value a block leaves behind
// is checked when the strip is written back.  Values and changes of honest training are orders of
// magnitude smaller, so a hit means the training has diverged; it raises a flag that the host
// reports as MF_ERANGE.  Both limits in the strip's scale (value * 2^24).
constexpr float kWatchValue = 1073741824.f;   // 2^30 = 64.0
constexpr float kWatchChange = 67108864.f;    // 2^26 =  4.0
constexpr float kWatchPlain = 64.f;           // the same value limit for numbers not yet scaled

struct RangeWatch {
    // per lane: the largest magnitudes seen (plain floats, kept in registers; compared once at
    // the end of the kernel)
    float value = 0.f, change = 0.f;           // in the strip's scale
    float plain = 0.f;                         // not scaled: values on their way into or out of the strip
    template <int VEC>
    __device__ __forceinline__ void see(const Row<VEC>& scaled_q, const Row<VEC>& scaled_dq)
    {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            value = fmaxf(value, fabsf(scaled_q.x[j]));
            change = fmaxf(change, fabsf(scaled_dq.x[j]));
        }
    }
    __device__ __forceinline__ void see_plain(float worst) { plain = fmaxf(plain, worst); }
    __device__ __forceinline__ bool hit() const
    {
        return !(plain < kWatchPlain) || !(value < kWatchValue) || !(change < kWatchChange);
    }
};

// EXACT = the strip holds fp32 bit patterns (deterministic mode), else fixed point (Hogwild).
template <typename T, int VEC, bool EXACT = false>
__device__ __forceinline__ Row<VEC> strip_read(const int* qrow, int lane, bool active)
{
    Row<VEC> q;
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        const int raw = active ? qrow[strip_elem<T>(lane, j)] : 0;
        q.x[j] = EXACT ? __int_as_float(raw) : from_fixed(raw);
    }
    return q;
}

// Calls f(0), f(1), ... f(N-1) with compile-time arguments until one returns false: a fully
// unrolled loop with an early exit whose register arrays keep constant indices.
template <class F, int... I>
__device__ __forceinline__ void unrolled_while(F&& f, std::integer_sequence<int, I...>)
{
    (void)(f(std::integral_constant<int, I>{}) && ...);
}
template <int N, class F>
__device__ __forceinline__ void unrolled_while(F&& f)
{
    unrolled_while(f, std::make_integer_sequence<int, N>{});
}

// The rows of P of the first DEPTH ratings of a batch, requested ahead of their use.
template <typename T, int K, int DEPTH>
struct RowRing {
    StoredRow<T, K> r[DEPTH];
};

template <typename T, int K, int DEPTH>
__device__ __forceinline__ RowRing<T, K, DEPTH> request_first_rows(const T* __restrict__ P, int mu, int cnt, int lane,
                                                                    bool active)
{
    RowRing<T, K, DEPTH> ring;
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        ring.r[d] = request_row<T, K, false>(P + (int64_t)uniform_lane(mu, min(d, cnt - 1)) * K, lane, active);
    return ring;
}

// Where the columns of a batch of ratings sit in the strip: lane l's column index becomes the
// index of that column's K values in LDS.  The strip holds either all columns of its range
// (slot = column - col0) or only the touched ones, packed (slots: one 16-bit entry per column of
// the range, written for the touched columns when the block began).
template <bool SPARSE>
__device__ __forceinline__ int strip_slots(int mv, int col0, const unsigned short* slots, bool valid)
{
    if constexpr (SPARSE) return valid ? (int)slots[mv - col0] : 0;
    else return mv - col0;
}

// A chunk whose rows of P belong to this wavefront alone.  Rows of P are cold (each is visited by
// one wavefront per launch), so their latency is hidden by requesting the row of the rating DEPTH
// positions ahead; every rating issues the same memory operations (one row request, one row
// store, whether or not the row changes) so that the wait counters are exact.  A rating whose row
// equals the previous rating's takes the row from registers: the request for it was issued before
// the previous ratings of that run were applied.  Requests past the end of the batch ask for its
// last row again; the unrolled group of DEPTH ratings in which the batch ends is left early.
// EXACT (deterministic mode, the wavefront is alone in its workgroup): the strip holds fp32, q_v
// is read and written in program order, every operation is the sequential order's.
template <typename T, int K, int DEPTH, bool EXACT, bool SPARSE>
__device__ __forceinline__ void lds_owned_chunk(T* __restrict__ P, int* strip, int col0, const unsigned short* slots,
                                                const int32_t* __restrict__ U,
                                                const int32_t* __restrict__ V,
                                                const float* __restrict__ R, int64_t begin,
                                                int32_t len, int mu, int mv, float mr,
                                                RowRing<T, K, DEPTH> first_rows, float lr,
                                                float shrink, int lane, bool active)
{
    // mu, mv, mr: the first batch of the chunk (rating `lane` of it), already loaded by the caller;
    // first_rows: the rows of P of its first DEPTH ratings, already requested by the caller
    constexpr int VEC = RowShape<T, K>::VEC;
    mv = strip_slots<SPARSE>(mv, col0, slots, lane < min(kWave, len));   // from here on: slots, not columns
    Row<VEC> p_prev;
#pragma unroll
    for (int j = 0; j < VEC; ++j) p_prev.x[j] = 0.f;
    int u_prev = -1;
    int nu = 0, nv = 0;
    float nr = 0.f;
    for (int32_t off = 0; off < len; off += kWave) {
        const int cnt = min(kWave, len - off);
        // the ratings of the batch after this one are requested now
        if (lane < len - off - kWave) {
            nu = U[begin + off + kWave + lane];
            nv = V[begin + off + kWave + lane];
            nr = R[begin + off + kWave + lane];
        }
        const int last = cnt - 1;
        StoredRow<T, K> ring[DEPTH];
        if (off == 0) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) ring[d] = first_rows.r[d];
        } else {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d)
                ring[d] = request_row<T, K, false>(P + (int64_t)uniform_lane(mu, min(d, last)) * K, lane, active);
        }
        int v_next = uniform_lane(mv, 0);
        Row<VEC> q_next = strip_read<T, VEC, EXACT>(strip + v_next * K, lane, active);
        // one rating: position d of its group of DEPTH, rating i of the batch; AHEAD: the row of
        // the rating DEPTH positions on is requested (not in the last, partial group of a batch)
        auto rating = [&](auto position, auto ahead, int i) {
                constexpr int d = decltype(position)::value;
                constexpr bool AHEAD = decltype(ahead)::value;
                const int u = uniform_lane(mu, i);
                const int v = v_next;
                const float r = __int_as_float(uniform_lane(__float_as_int(mr), i));
                const Row<VEC> arrived = row_values<T, K>(ring[d]);
                Row<VEC> p;
#pragma unroll
                for (int j = 0; j < VEC; ++j) p.x[j] = (u == u_prev) ? p_prev.x[j] : arrived.x[j];
                if constexpr (AHEAD)
                    ring[d] = request_row<T, K, false>(P + (int64_t)uniform_lane(mu, min(i + DEPTH, last)) * K, lane, active);
                const Row<VEC> q = q_next;
                int* const qrow = strip + v * K;
                v_next = uniform_lane(mv, min(i + 1, last));
                const Row<VEC> q_ahead = strip_read<T, VEC, EXACT>(strip + v_next * K, lane, active);
                float e;
                if constexpr (EXACT && sizeof(T) == 2) {
                    double part = 0.0;   // see sgd_chunks: the binary16 result must not depend on summation order
#pragma unroll
                    for (int j = 0; j < VEC; ++j) part = fma((double)p.x[j], (double)q.x[j], part);
                    e = r - (float)wave_sum_f64_dpp(part);
                } else {
                    float part = 0.f;
#pragma unroll
                    for (int j = 0; j < VEC; ++j) part = fmaf(p.x[j], q.x[j], part);
                    e = r - wave_sum(part);
                }
                const float step = lr * e;
                const float sh = shrink;
                Row<VEC> p2;
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    p2.x[j] = quantise<T>(p.x[j] + fmaf(step, q.x[j], -sh * p.x[j]));
                    // the read-ahead of the next column was taken before this column is changed
                    if constexpr (EXACT) {
                        const float q2 = quantise<T>(q.x[j] + fmaf(step, p.x[j], -sh * q.x[j]));
                        if (active) qrow[strip_elem<T>(lane, j)] = __float_as_int(q2);
                        q_next.x[j] = (v_next == v) ? q2 : q_ahead.x[j];
                    } else {
                        const int dq = to_fixed(fmaf(step, p.x[j], -sh * q.x[j]));
                        if (active) atomicAdd(&qrow[strip_elem<T>(lane, j)], dq);
                        q_next.x[j] = (v_next == v) ? q.x[j] + from_fixed(dq) : q_ahead.x[j];
                    }
                }
                store_row<VEC>(P + (int64_t)u * K, lane, active, p2);
                p_prev = p2;
                u_prev = u;
        };
        // whole groups of DEPTH ratings: the same memory operations at every position, so the wait
        // counts are static; then what is left of the batch, with an exit after every rating
        int base = 0;
        for (; base + DEPTH <= cnt; base += DEPTH)
            unrolled_while<DEPTH>([&](auto position) {
                rating(position, std::true_type{}, base + decltype(position)::value);
                return true;
            });
        unrolled_while<DEPTH - 1>([&](auto position) {
            const int i = base + decltype(position)::value;
            if (i >= cnt) return false;
            rating(position, std::false_type{}, i);
            return true;
        });
        mu = nu;
        mv = strip_slots<SPARSE>(nv, col0, slots, lane < len - off - kWave);
        mr = nr;
    }
}

// ---- Hogwild version of the loop above, trimmed for instruction count -------------------------
// With 16 wavefronts per compute unit this loop is bound by VALU issue (measured: 0.245 us per
// rating and wavefront = 37 cycles per rating and compute unit at ~50 VALU instructions), so:
//  * q_v is kept in the scale of its fixed-point strip (float(q_fixed) = q * 2^24): reading it is
//    one conversion, the change is one fused multiply-add and one conversion, and the factor
//    2^-24 moves into the two wave-uniform step sizes;
//  * the next rating's column is read from LDS AFTER this rating's atomic add (LDS executes a
//    wavefront's operations in order), so no forwarding is needed when the column repeats; the
//    read's latency is covered by the other wavefronts of the SIMD;
//  * p_u is updated with two fused operations (the extra rounding of the deterministic form is
//    irrelevant here);
//  * the last two steps of the cross-lane sum are single DPP adds.
__device__ __forceinline__ float wave_sum_fused(float x)
{
    x = dpp_add<0xB1, 0xf>(x);
    x = dpp_add<0x4E, 0xf>(x);
    x = dpp_add<0x141, 0xf>(x);
    x = dpp_add<0x140, 0xf>(x);
    // rows 1 and 3 add lane 15 of the row before; then rows 2 and 3 add lane 31: one instruction
    // each (rows outside the mask keep their value); two wait states before a DPP read
    asm("s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf" : "+v"(x));
    asm("s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf" : "+v"(x));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

template <typename T, int K, int DEPTH, bool SPARSE>
__device__ __forceinline__ void lds_hog_chunk(T* __restrict__ P, int* strip, int col0, const unsigned short* slots,
                                              const int32_t* __restrict__ U,
                                              const int32_t* __restrict__ V,
                                              const float* __restrict__ R, int64_t begin, int32_t len,
                                              int mu, int mv, float mr,
                                              RowRing<T, K, DEPTH> first_rows, float lr,
                                              float shrink, int lane, bool active, RangeWatch& watch)
{
    constexpr int VEC = RowShape<T, K>::VEC;
    mv = strip_slots<SPARSE>(mv, col0, slots, lane < min(kWave, len));   // from here on: slots, not columns
    Row<VEC> p_prev;
#pragma unroll
    for (int j = 0; j < VEC; ++j) p_prev.x[j] = 0.f;
    int u_prev = -1;
    int nu = 0, nv = 0;
    float nr = 0.f;
    auto row_of = [&](int u) { return P + (int64_t)u * K; };
    auto read_scaled = [&](int slot) {
        const int* qrow = strip + slot * K;
        Row<VEC> q;
#pragma unroll
        for (int j = 0; j < VEC; ++j) q.x[j] = active ? (float)qrow[strip_elem<T>(lane, j)] : 0.f;
        return q;
    };
    const int quarter = len >> 2, half = len >> 1, three_quarters = half + quarter;
    for (int32_t off = 0; off < len; off += kWave) {
        const int cnt = min(kWave, len - off);
        if (lane < len - off - kWave) {
            nu = U[begin + off + kWave + lane];
            nv = V[begin + off + kWave + lane];
            nr = R[begin + off + kWave + lane];
        }
        const int last = cnt - 1;
        StoredRow<T, K> ring[DEPTH];
        if (off == 0) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) ring[d] = first_rows.r[d];
        } else {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d)
                ring[d] = request_row<T, K, false>(row_of(uniform_lane(mu, min(d, last))), lane, active);
        }
        Row<VEC> qs = read_scaled(uniform_lane(mv, 0));
        // one rating: position d of its group of DEPTH, rating i of the batch; AHEAD: the row of
        // the rating DEPTH positions on is requested (not in the last, partial group of a batch)
        auto rating = [&](auto position, auto ahead, int i) {
            constexpr int d = decltype(position)::value;
            constexpr bool AHEAD = decltype(ahead)::value;
            const int u = uniform_lane(mu, i);
            const int v = uniform_lane(mv, i);
            const float r = __int_as_float(uniform_lane(__float_as_int(mr), i));
            const Row<VEC> arrived = row_values<T, K>(ring[d]);
            Row<VEC> p;
#pragma unroll
            for (int j = 0; j < VEC; ++j) p.x[j] = (u == u_prev) ? p_prev.x[j] : arrived.x[j];
            if constexpr (AHEAD)
                ring[d] = request_row<T, K, false>(row_of(uniform_lane(mu, min(i + DEPTH, last))), lane, active);
            float part = 0.f;
#pragma unroll
            for (int j = 0; j < VEC; ++j) part = fmaf(p.x[j], qs.x[j], part);
            const float e = fmaf(-kFromFixed, wave_sum_fused(part), r);
            const float step = lr * e;
            const float step_q = step * kFromFixed;   // (lr*e) * q       = step_q * qs
            const float step_p = step * kToFixed;     // (lr*e) * p * 2^24 = step_p * p
            int* const qrow = strip + v * K;
            Row<VEC> p2, dqs;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                p2.x[j] = quantise<T>(fmaf(step_q, qs.x[j], fmaf(-shrink, p.x[j], p.x[j])));
                dqs.x[j] = fmaf(step_p, p.x[j], -shrink * qs.x[j]);
                const int dq = __float2int_rn(dqs.x[j]);
                if (active) atomicAdd(&qrow[strip_elem<T>(lane, j)], dq);
            }
            watch.see<VEC>(qs, dqs);
            store_row<VEC>(row_of(u), lane, active, p2);
            qs = read_scaled(uniform_lane(mv, min(i + 1, last)));   // after the add above
            p_prev = p2;
            u_prev = u;
        };
        // whole groups of DEPTH ratings: the same memory operations at every position, so the wait
        // counts are static; then what is left of the batch, with an exit after every rating
        int base = 0;
        for (; base + DEPTH <= cnt; base += DEPTH) {
            // The wavefronts of a workgroup get equal shares of the block, but the instruction
            // arbiter favours the oldest wavefront of a SIMD: left alone they finish one after
            // the other and the last ones run alone, far below the issue rate.  A wavefront with
            // more of its chunk left asks for a higher priority, which keeps them level.
            // Only in the build with the long prefetch depth, which is the one taken for large
            // inputs: on short chunks the priority changes were measured to cost 2 %.
            if constexpr (DEPTH > kShortPrefetchDepth) {
                const int left = len - off - base;
                if (left > three_quarters) __builtin_amdgcn_s_setprio(3);
                else if (left > half) __builtin_amdgcn_s_setprio(2);
                else if (left > quarter) __builtin_amdgcn_s_setprio(1);
                else __builtin_amdgcn_s_setprio(0);
            }
            unrolled_while<DEPTH>([&](auto position) {
                rating(position, std::true_type{}, base + decltype(position)::value);
                return true;
            });
        }
        if constexpr (DEPTH > kShortPrefetchDepth) {
            if (base < cnt) __builtin_amdgcn_s_setprio(0);
        }
        unrolled_while<DEPTH - 1>([&](auto position) {
            const int i = base + decltype(position)::value;
            if (i >= cnt) return false;
            rating(position, std::false_type{}, i);
            return true;
        });
        mu = nu;
        mv = strip_slots<SPARSE>(nv, col0, slots, lane < len - off - kWave);
        mr = nr;
    }
    if constexpr (DEPTH > kShortPrefetchDepth) __builtin_amdgcn_s_setprio(0);
}

// ---- rows of P cut by entry boundaries, held in LDS while their block runs ----------------------
// A very long row is shared out over several wavefronts of the workgroup.  Its p_u then lives in
// LDS beside the strip, in the strip's fixed-point format, for as long as the block runs, and is
// read and changed exactly like q_v (LDS atomic adds: no change is lost, every wavefront sees the
// others' changes at once).  `prow`: the row's LDS slot.  All ratings of the piece have this row.
// Both operands stay in the strip's scale (see lds_hog_chunk), and the operands of the NEXT rating
// are read from LDS before this rating's sum is reduced: LDS executes a wavefront's operations in
// order, so those reads see the state before this rating's own adds, which are then applied to
// the copies in registers (changes other wavefronts make meanwhile arrive one rating later).
template <typename T, int K, bool SPARSE>
__device__ __forceinline__ void lds_hot_row_piece(int* prow, int* strip, int col0, const unsigned short* slots,
                                                  const int32_t* __restrict__ V,
                                                  const float* __restrict__ R, int64_t begin, int32_t len,
                                                  float lr, float shrink, int lane, bool active, RangeWatch& watch)
{
    constexpr int VEC = RowShape<T, K>::VEC;
    constexpr float kFromFixedSquared = kFromFixed * kFromFixed;
    auto read_scaled = [&](const int* row) {
        Row<VEC> x;
#pragma unroll
        for (int j = 0; j < VEC; ++j) x.x[j] = active ? (float)row[strip_elem<T>(lane, j)] : 0.f;
        return x;
    };
    int mv = 0, nv = 0;
    float mr = 0.f, nr = 0.f;
    if (lane < min(kWave, len)) {
        mv = V[begin + lane];
        mr = R[begin + lane];
    }
    mv = strip_slots<SPARSE>(mv, col0, slots, lane < min(kWave, len));   // slots, not columns
    Row<VEC> qs = read_scaled(strip + uniform_lane(mv, 0) * K);
    Row<VEC> ps = read_scaled(prow);
    for (int32_t off = 0; off < len; off += kWave) {
        const int cnt = min(kWave, len - off);
        const bool more = len - off > kWave;
        if (lane < len - off - kWave) {
            nv = V[begin + off + kWave + lane];
            nr = R[begin + off + kWave + lane];
        }
        for (int i = 0; i < cnt; ++i) {
            const int v = uniform_lane(mv, i);
            const float r = __int_as_float(uniform_lane(__float_as_int(mr), i));
            int* const qrow = strip + v * K;
            // the column of the rating after this one (at the end of the piece: this one again)
            const int v_next = i + 1 < cnt ? uniform_lane(mv, i + 1)
                                           : (more ? strip_slots<SPARSE>(uniform_lane(nv, 0), col0, slots, true) : v);
            Row<VEC> qn = read_scaled(strip + v_next * K);
            Row<VEC> pn = read_scaled(prow);
            float part = 0.f;
#pragma unroll
            for (int j = 0; j < VEC; ++j) part = fmaf(ps.x[j], qs.x[j], part);
            const float step = lr * fmaf(-kFromFixedSquared, wave_sum_fused(part), r);
            Row<VEC> dqs, dps;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                dqs.x[j] = fmaf(step, ps.x[j], -shrink * qs.x[j]);
                dps.x[j] = fmaf(step, qs.x[j], -shrink * ps.x[j]);
                const int dq = __float2int_rn(dqs.x[j]);
                const int dp = __float2int_rn(dps.x[j]);
                if (active) {
                    atomicAdd(&qrow[strip_elem<T>(lane, j)], dq);
                    atomicAdd(&prow[strip_elem<T>(lane, j)], dp);
                }
                pn.x[j] += (float)dp;
                if (v_next == v) qn.x[j] += (float)dq;
            }
            watch.see<VEC>(qs, dqs);
            watch.see<VEC>(ps, dps);
            qs = qn;
            ps = pn;
        }
        mv = strip_slots<SPARSE>(nv, col0, slots, lane < len - off - kWave);
        mr = nr;
    }
}

// Number of ratings at the front (FROM_END: at the back) of the packed range [begin, begin+len)
// whose row index is `u`; wave-uniform.
template <bool FROM_END>
__device__ __forceinline__ int32_t run_of_row(const int32_t* __restrict__ U, int64_t begin, int32_t len, int u,
                                              int lane)
{
    int32_t run = 0;
    for (int32_t off = 0; off < len; off += kWave) {
        const int cnt = min(kWave, len - off);
        const int64_t at = FROM_END ? begin + len - 1 - off - lane : begin + off + lane;
        const bool same = lane < cnt && U[at] == u;
        const unsigned long long others = ~__ballot(same);   // lanes past cnt count as "another row"
        const int first_other = others ? __builtin_ctzll(others) : kWave;
        run += min(first_other, cnt);
        if (first_other < cnt) break;
    }
    return run;
}

typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));
constexpr int kRawBufferFlags = 0x00020000;   // word 3 of a raw (untyped, unswizzled) buffer descriptor on gfx9
constexpr int kCachePolicySc1 = 16;           // auxiliary operand of the buffer intrinsics: bit 4 = sc1

// ---- the strip of Qt in LDS -------------------------------------------------------------------
// COHERENT: the strip is handed from workgroup to workgroup INSIDE one launch (ring kernel
// below), possibly across dies whose L2s do not see each other's plain stores; it is then read
// and written with agent-scope accesses (sc1: past the L2s' non-coherent lines).
// Values entering and leaving the fixed-point strip are watched (a value of magnitude >= 128
// saturates on entry): each copy keeps a running maximum of the magnitudes that passed.
// `worst`: the caller's running maximum of the magnitudes that passed (see RangeWatch).
template <bool EXACT>
__device__ __forceinline__ int to_strip(float x, float& worst)
{
    if constexpr (EXACT) return __float_as_int(x);
    worst = fmaxf(worst, fabsf(x));
    return to_fixed(x);
}

template <bool EXACT>
__device__ __forceinline__ float from_strip(int x, float& worst)
{
    if constexpr (EXACT) return __int_as_float(x);
    const float f = from_fixed(x);
    worst = fmaxf(worst, fabsf(f));
    return f;
}

// SPARSE (the one-launch Hogwild form, where a wavefront's 64 consecutive words of a strip lie in
// one column): the LDS holds only the columns of the strip in which the block has a rating,
// packed in ascending order -- the s-th touched column in slot s -- so a strip may span more
// columns than the LDS could hold.  The block's table of touched columns (one bit per column of
// the strip's range) comes with lane l of every wavefront holding bit word l (`mask_word`).
template <typename T, int K>
struct SparseStrip {
    static constexpr int kWordsPerColumn = K * (int)sizeof(T) / 4;
    static constexpr bool kPossible = kWordsPerColumn % kWave == 0;
};

// What a wavefront needs to move its share of a packed strip.  The columns' values are moved in
// pieces of 64 consecutive 32-bit words of the strip's range in memory; piece j of a wavefront
// begins at word (its first thread) + j * blockDim.x.  `pieces`: bit j set = piece j lies in a
// touched column; `piece_slot`: lane j holds that column's slot.  `first_slot`: lane l holds the
// slot of the first touched column of bit word l; `n_slots`: touched columns in all.  Worked out
// once per block by the 64 lanes together.  Needs words <= 64 * blockDim.x and all lanes active.
struct StripMap {
    unsigned long long pieces;
    int piece_slot;
    int first_slot;
    int n_slots;
    unsigned mask;    // lane l: bit word l of the block's table
};

// The touched columns of a strip one after the other, in ascending order (wave-uniform; for the
// one-wavefront workgroups of the deterministic form, which move a strip column by column).
struct TouchedColumns {
    unsigned mask;    // lane l: bit word l
    int n_words;
    int word;
    unsigned bits;
    __device__ __forceinline__ TouchedColumns(unsigned mask_, int ncols) : mask(mask_), n_words((ncols + 31) >> 5), word(0)
    {
        bits = n_words > 0 ? (unsigned)uniform_lane((int)mask, 0) : 0u;
    }
    __device__ __forceinline__ int next()   // the next touched column (offset in the strip's range), or -1
    {
        while (bits == 0u && word + 1 < n_words) {
            word += 1;
            bits = (unsigned)uniform_lane((int)mask, word);
        }
        if (bits == 0u) return -1;
        const int bit = __builtin_ctz(bits);
        bits &= bits - 1u;
        return 32 * word + bit;
    }
};

// How the one wavefront of a deterministic workgroup holds a column of K values in memory: lane l
// has kWords consecutive 32-bit words from word l * kWords on; lanes >= kLanes are idle.
template <typename T, int K>
struct ColumnShape {
    static constexpr int kColumnWords = K * (int)sizeof(T) / 4;
    static constexpr int kWords = kColumnWords >= kWave ? kColumnWords / kWave : 1;
    static constexpr int kLanes = kColumnWords / kWords;
    static constexpr int kPerWord = sizeof(T) == 2 ? 2 : 1;    // values per word
};

template <typename T, int K>
__device__ __forceinline__ StripMap map_strip(int ncols, unsigned mask_word)
{
    const int lane = threadIdx.x & (kWave - 1);
    StripMap m;
    const int mine = __popc(mask_word);
    int upto = mine;                         // touched columns in bit words 0 .. lane
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int below = __shfl_up(upto, d, kWave);
        if (lane >= d) upto += below;
    }
    m.mask = mask_word;
    m.first_slot = upto - mine;
    m.n_slots = uniform_lane(upto, kWave - 1);
    const int words = ncols * SparseStrip<T, K>::kWordsPerColumn;
    const int w = (int)(threadIdx.x & ~(unsigned)(kWave - 1)) + lane * (int)blockDim.x;
    const int column = min(w, words - 1) / SparseStrip<T, K>::kWordsPerColumn;
    const unsigned bits = (unsigned)__shfl((int)mask_word, column >> 5, kWave);
    const int before = __shfl(m.first_slot, column >> 5, kWave);
    m.piece_slot = before + __popc(bits & ((1u << (column & 31)) - 1u));
    m.pieces = __ballot(w < words && ((bits >> (column & 31)) & 1u));
    return m;
}

// The 16-bit table column -> slot that the wavefronts' chunks look their columns up in: written
// for the touched columns of the range, each bit word by one wavefront.
__device__ __forceinline__ void write_slot_table(unsigned short* slots, unsigned mask_word, const StripMap& m)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = (int)(threadIdx.x >> 6), n_waves = (int)(blockDim.x >> 6);
    unsigned left = (lane % n_waves == wave) ? mask_word : 0u;
    int slot = m.first_slot;
    while (left) {
        const int bit = __builtin_ctz(left);
        left &= left - 1u;
        slots[32 * lane + bit] = (unsigned short)slot++;
    }
}

// Columns col0 .. col0+ncols of Qt into LDS, by all threads of the workgroup (no barrier inside).
template <typename T, int K, bool EXACT, bool COHERENT, bool SPARSE>
__device__ __forceinline__ void strip_copy_in(int* strip, const T* __restrict__ Qt, int col0, int ncols,
                                              RangeWatch& watch, const StripMap& map)
{
    float worst = 0.f;
    const int total = ncols * K;          // multiple of 32
    const T* const strip_src = Qt + (int64_t)col0 * K;
    const int stride = 4 * (int)blockDim.x;
    if constexpr (EXACT && SPARSE) {
        // one wavefront: the touched columns one after the other into consecutive slots, eight
        // columns requested, then stored
        using Shape = ColumnShape<T, K>;
        const int lane = threadIdx.x & (kWave - 1);
        const unsigned* src = reinterpret_cast<const unsigned*>(strip_src);
        constexpr int kInFlight = 8;
        TouchedColumns columns(map.mask, ncols);
        int slot = 0;
        for (;;) {
            int col[kInFlight];
            int n = 0;
#pragma unroll
            for (int t = 0; t < kInFlight; ++t) {
                col[t] = columns.next();
                if (col[t] >= 0) n = t + 1;
            }
            if (n == 0) break;
            unsigned raw[kInFlight][Shape::kWords];
#pragma unroll
            for (int t = 0; t < kInFlight; ++t)
                if (t < n && lane < Shape::kLanes) {
#pragma unroll
                    for (int j = 0; j < Shape::kWords; ++j)
                        raw[t][j] = load_word<COHERENT>(src + col[t] * Shape::kColumnWords + lane * Shape::kWords + j);
                }
#pragma unroll
            for (int t = 0; t < kInFlight; ++t)
                if (t < n && lane < Shape::kLanes) {
#pragma unroll
                    for (int j = 0; j < Shape::kWords; ++j) {
                        int* at = strip + (slot + t) * K + (lane * Shape::kWords + j) * Shape::kPerWord;
                        if constexpr (sizeof(T) == 2) {
                            const float2 f = unpack_half2(raw[t][j]);
                            at[0] = to_strip<EXACT>(f.x, worst);
                            at[1] = to_strip<EXACT>(f.y, worst);
                        } else {
                            at[0] = to_strip<EXACT>(__uint_as_float(raw[t][j]), worst);
                        }
                    }
                }
            slot += n;
        }
    } else if constexpr (!EXACT && SPARSE) {
        // the touched columns only, into their slots: up to 16 pieces requested, then converted
        constexpr int kPerWord = sizeof(T) == 2 ? 2 : 1;
        constexpr int kInColumn = SparseStrip<T, K>::kWordsPerColumn - 1;
        const unsigned* src = reinterpret_cast<const unsigned*>(strip_src);
        constexpr int kInFlight = 16;
        unsigned long long left = map.pieces;
        while (left) {
            const int n = min(kInFlight, (int)__popcll(left));
            unsigned raw[kInFlight];
            int at[kInFlight];
#pragma unroll
            for (int t = 0; t < kInFlight; ++t) {
                if (t < n) {
                    const int j = __builtin_ctzll(left);
                    left &= left - 1ull;
                    const int w = (int)threadIdx.x + j * (int)blockDim.x;
                    at[t] = uniform_lane(map.piece_slot, j) * K + (w & kInColumn) * kPerWord;
                    raw[t] = load_word<COHERENT>(src + w);
                }
            }
#pragma unroll
            for (int t = 0; t < kInFlight; ++t) {
                if (t < n) {
                    if constexpr (sizeof(T) == 2) {
                        const float2 f = unpack_half2(raw[t]);
                        strip[at[t]] = to_strip<EXACT>(f.x, worst);
                        strip[at[t] + 1] = to_strip<EXACT>(f.y, worst);
                    } else {
                        strip[at[t]] = to_strip<EXACT>(__uint_as_float(raw[t]), worst);
                    }
                }
            }
        }
    } else if constexpr (COHERENT && !EXACT) {
        // 1024 threads: one 32-bit word each (one fp32 value or one pair of binary16 values); wider
        // pieces were measured slower here, and faster for the 64-thread workgroups of the
        // deterministic mode below
        constexpr int kPerWord = sizeof(T) == 2 ? 2 : 1;
        const unsigned* src = reinterpret_cast<const unsigned*>(strip_src);
        const int words = total / kPerWord;
        constexpr int kInFlight = 16;
        for (int w0 = (int)threadIdx.x; w0 < words; w0 += kInFlight * (int)blockDim.x) {
            unsigned raw[kInFlight];
#pragma unroll
            for (int t = 0; t < kInFlight; ++t) {
                const int w = w0 + t * (int)blockDim.x;
                if (w < words) raw[t] = load_word<true>(src + w);
            }
#pragma unroll
            for (int t = 0; t < kInFlight; ++t) {
                const int w = w0 + t * (int)blockDim.x;
                if (w < words) {
                    if constexpr (sizeof(T) == 2) {
                        const float2 f = unpack_half2(raw[t]);
                        strip[2 * w] = to_strip<EXACT>(f.x, worst);
                        strip[2 * w + 1] = to_strip<EXACT>(f.y, worst);
                    } else {
                        strip[w] = to_strip<EXACT>(__uint_as_float(raw[t]), worst);
                    }
                }
            }
        }
    } else if constexpr (COHERENT) {
        // 16-byte pieces (4 fp32 values or 8 binary16 values) through a raw buffer descriptor of
        // the strip with the agent-scope cache policy (sc1)
        constexpr int kPerPiece = 16 / (int)sizeof(T);
        const int pieces = total / kPerPiece;
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc((void*)strip_src, 0, total * (int)sizeof(T), kRawBufferFlags);
        constexpr int kInFlight = 16;
        for (int p0 = (int)threadIdx.x; p0 < pieces; p0 += kInFlight * (int)blockDim.x) {
            uint4_t raw[kInFlight];
#pragma unroll
            for (int t = 0; t < kInFlight; ++t) {
                const int pc = p0 + t * (int)blockDim.x;
                if (pc < pieces) raw[t] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, pc * 16, 0, kCachePolicySc1);
            }
#pragma unroll
            for (int t = 0; t < kInFlight; ++t) {
                const int pc = p0 + t * (int)blockDim.x;
                if (pc < pieces) {
                    if constexpr (sizeof(T) == 2) {
#pragma unroll
                        for (int h = 0; h < 4; ++h) {
                            const float2 f = unpack_half2(raw[t][h]);
                            strip[pc * 8 + 2 * h] = to_strip<EXACT>(f.x, worst);
                            strip[pc * 8 + 2 * h + 1] = to_strip<EXACT>(f.y, worst);
                        }
                    } else {
                        *reinterpret_cast<int4*>(strip + pc * 4) =
                            make_int4(to_strip<EXACT>(__uint_as_float(raw[t][0]), worst),
                                      to_strip<EXACT>(__uint_as_float(raw[t][1]), worst),
                                      to_strip<EXACT>(__uint_as_float(raw[t][2]), worst),
                                      to_strip<EXACT>(__uint_as_float(raw[t][3]), worst));
                    }
                }
            }
        }
    } else {
        constexpr int kInFlight = 8;   // loads of the strip copy each thread keeps in flight
        for (int i0 = 4 * (int)threadIdx.x; i0 < total; i0 += kInFlight * stride) {
            float4 val[kInFlight];
#pragma unroll
            for (int t = 0; t < kInFlight; ++t) {
                const int i = i0 + t * stride;
                if (i < total) {
                    if constexpr (sizeof(T) == 2) {
                        uint2 raw = *reinterpret_cast<const uint2*>(strip_src + i);
                        float2 a = unpack_half2(raw.x), b = unpack_half2(raw.y);
                        val[t] = make_float4(a.x, a.y, b.x, b.y);
                    } else {
                        val[t] = *reinterpret_cast<const float4*>(strip_src + i);
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < kInFlight; ++t) {
                const int i = i0 + t * stride;
                if (i < total)
                    *reinterpret_cast<int4*>(strip + i) =
                        make_int4(to_strip<EXACT>(val[t].x, worst), to_strip<EXACT>(val[t].y, worst),
                                  to_strip<EXACT>(val[t].z, worst), to_strip<EXACT>(val[t].w, worst));
            }
        }
    }
    if constexpr (!EXACT) watch.see_plain(worst);
}

// The strip in LDS back to columns col0 .. col0+ncols of Qt, by all threads of the workgroup.
template <typename T, int K, bool EXACT, bool COHERENT, bool SPARSE>
__device__ __forceinline__ void strip_copy_out(const int* strip, T* __restrict__ Qt, int col0, int ncols,
                                               RangeWatch& watch, const StripMap& map)
{
    float worst = 0.f;
    const int total = ncols * K;
    T* const strip_dst = Qt + (int64_t)col0 * K;
    const int stride = 4 * (int)blockDim.x;
    if constexpr (EXACT && SPARSE) {
        using Shape = ColumnShape<T, K>;
        const int lane = threadIdx.x & (kWave - 1);
        unsigned* dst = reinterpret_cast<unsigned*>(strip_dst);
        TouchedColumns columns(map.mask, ncols);
        int slot = 0;
        for (int col = columns.next(); col >= 0; col = columns.next(), ++slot) {
            if (lane < Shape::kLanes) {
#pragma unroll
                for (int j = 0; j < Shape::kWords; ++j) {
                    const int* at = strip + slot * K + (lane * Shape::kWords + j) * Shape::kPerWord;
                    unsigned raw;
                    if constexpr (sizeof(T) == 2) {
                        __half2 h = __halves2half2(round_to_half(from_strip<EXACT>(at[0], worst)),
                                                   round_to_half(from_strip<EXACT>(at[1], worst)));
                        raw = *reinterpret_cast<unsigned*>(&h);
                    } else {
                        raw = __float_as_uint(from_strip<EXACT>(at[0], worst));
                    }
                    unsigned* to = dst + col * Shape::kColumnWords + lane * Shape::kWords + j;
                    if constexpr (COHERENT) __hip_atomic_store(to, raw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    else *to = raw;
                }
            }
        }
    } else if constexpr (!EXACT && SPARSE) {
        constexpr int kPerWord = sizeof(T) == 2 ? 2 : 1;
        constexpr int kInColumn = SparseStrip<T, K>::kWordsPerColumn - 1;
        unsigned* dst = reinterpret_cast<unsigned*>(strip_dst);
        unsigned long long left = map.pieces;
        while (left) {
            const int j = __builtin_ctzll(left);
            left &= left - 1ull;
            const int w = (int)threadIdx.x + j * (int)blockDim.x;
            const int at = uniform_lane(map.piece_slot, j) * K + (w & kInColumn) * kPerWord;
            unsigned raw;
            if constexpr (sizeof(T) == 2) {
                __half2 h = __halves2half2(round_to_half(from_strip<EXACT>(strip[at], worst)),
                                           round_to_half(from_strip<EXACT>(strip[at + 1], worst)));
                raw = *reinterpret_cast<unsigned*>(&h);
            } else {
                raw = __float_as_uint(from_strip<EXACT>(strip[at], worst));
            }
            if constexpr (COHERENT) __hip_atomic_store(dst + w, raw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else dst[w] = raw;
        }
    } else if constexpr (COHERENT && !EXACT) {
        constexpr int kPerWord = sizeof(T) == 2 ? 2 : 1;
        unsigned* dst = reinterpret_cast<unsigned*>(strip_dst);
        const int words = total / kPerWord;
        for (int w = (int)threadIdx.x; w < words; w += (int)blockDim.x) {
            unsigned raw;
            if constexpr (sizeof(T) == 2) {
                __half2 h = __halves2half2(round_to_half(from_strip<EXACT>(strip[2 * w], worst)),
                                           round_to_half(from_strip<EXACT>(strip[2 * w + 1], worst)));
                raw = *reinterpret_cast<unsigned*>(&h);
            } else {
                raw = __float_as_uint(from_strip<EXACT>(strip[w], worst));
            }
            __hip_atomic_store(dst + w, raw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    } else if constexpr (COHERENT) {
        constexpr int kPerPiece = 16 / (int)sizeof(T);
        const int pieces = total / kPerPiece;
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc((void*)strip_dst, 0, total * (int)sizeof(T), kRawBufferFlags);
        for (int pc = (int)threadIdx.x; pc < pieces; pc += (int)blockDim.x) {
            uint4_t raw;
            if constexpr (sizeof(T) == 2) {
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    __half2 hh = __halves2half2(round_to_half(from_strip<EXACT>(strip[pc * 8 + 2 * h], worst)),
                                                round_to_half(from_strip<EXACT>(strip[pc * 8 + 2 * h + 1], worst)));
                    raw[h] = *reinterpret_cast<unsigned*>(&hh);
                }
            } else {
                const int4 v = *reinterpret_cast<const int4*>(strip + pc * 4);
                raw[0] = __float_as_uint(from_strip<EXACT>(v.x, worst));
                raw[1] = __float_as_uint(from_strip<EXACT>(v.y, worst));
                raw[2] = __float_as_uint(from_strip<EXACT>(v.z, worst));
                raw[3] = __float_as_uint(from_strip<EXACT>(v.w, worst));
            }
            __builtin_amdgcn_raw_buffer_store_b128(raw, rsrc, pc * 16, 0, kCachePolicySc1);
        }
    } else {
        for (int i = 4 * (int)threadIdx.x; i < total; i += stride) {
            const int4 raw4 = *reinterpret_cast<const int4*>(strip + i);
            const float4 val = make_float4(from_strip<EXACT>(raw4.x, worst), from_strip<EXACT>(raw4.y, worst),
                                           from_strip<EXACT>(raw4.z, worst), from_strip<EXACT>(raw4.w, worst));
            if constexpr (sizeof(T) == 2) {
                __half2 a = __halves2half2(round_to_half(val.x), round_to_half(val.y));
                __half2 b = __halves2half2(round_to_half(val.z), round_to_half(val.w));
                uint2 raw;
                raw.x = *reinterpret_cast<unsigned*>(&a);
                raw.y = *reinterpret_cast<unsigned*>(&b);
                *reinterpret_cast<uint2*>(strip_dst + i) = raw;
            } else {
                *reinterpret_cast<float4*>(strip_dst + i) = val;
            }
        }
    }
    if constexpr (!EXACT) watch.see_plain(worst);
}

// Work of one workgroup on one block: copy the strip in, run the block's entries, copy it back.
// `before_strip()` is called after the block's first ratings and rows of P have been requested
// and before the strip is read: the ring kernel waits there for the strip's previous user
// (returning false means "give up": the workgroup leaves); everything requested before it is
// independent of the strip.  copy_in / copy_out = false: the caller moves the strip itself.
template <typename T, int K, bool EXACT, bool COHERENT, int DEPTH, bool SPARSE, class BeforeStrip>
__device__ __forceinline__ bool lds_block_body(int* strip, T* __restrict__ P, T* __restrict__ Qt,
                                               const int32_t* __restrict__ U, const int32_t* __restrict__ V,
                                               const float* __restrict__ R,
                                               const int64_t* __restrict__ entry_begin,
                                               const int32_t* __restrict__ entry_len,
                                               const int64_t* __restrict__ hot_pos, const LdsBlock blk,
                                               float lr, float lambda, bool copy_in, bool copy_out, unsigned mask_word,
                                               int slot_table_at, RangeWatch& watch, BeforeStrip before_strip)
{
    const int lane = threadIdx.x & (kWave - 1);
    const bool active = RowShape<T, K>::ACTIVE == kWave ? true : lane < RowShape<T, K>::ACTIVE;
    int total = blk.ncols * K;                // values of the strip in LDS (SPARSE: set below); multiple of 32

    // Entries are dealt to the wavefronts round-robin.  The first entry's ratings are requested
    // before the strip is copied so that the two latencies overlap.
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = (int)(blockDim.x >> 6);
    int32_t raw_len = 0;
    int64_t begin = 0;
    int mu = 0, mv = 0;
    float mr = 0.f;
    auto fetch_entry = [&](int e) {
        raw_len = entry_len[blk.first_entry + e];
        begin = entry_begin[blk.first_entry + e];
        if (lane < min(kWave, raw_len & ~kSharedRowFlag)) {
            mu = U[begin + lane];
            mv = V[begin + lane];
            mr = R[begin + lane];
        }
    };
    constexpr int VEC = RowShape<T, K>::VEC;
    // rows of P cut by the entry boundaries of this block: lane s of every wavefront knows the
    // row index of slot s; the slots follow the strip in LDS
    const int n_hot = EXACT ? 0 : (blk.hot & 15);
    int hot_u = -1;
    if (!EXACT && lane < n_hot) hot_u = U[hot_pos[(blk.hot >> 4) + lane]];
    RowRing<T, K, DEPTH> first_rows;
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
#pragma unroll
        for (int j = 0; j < StoredRow<T, K>::WORDS; ++j) first_rows.r[d].w[j] = 0u;
    if (wave < blk.n_entries) {
        fetch_entry(wave);
        if (EXACT || raw_len > 0)
            first_rows = request_first_rows<T, K, DEPTH>(P, mu, min(kWave, raw_len & ~kSharedRowFlag), lane,
                                                                     active);
    }
    if (!before_strip()) return false;

    // SPARSE: where the touched columns go in LDS, and the table the chunks look columns up in
    // (at a fixed place behind the values; nobody reads the previous block's table any more)
    StripMap map{};
    unsigned short* slots = nullptr;
    if constexpr (SPARSE) {
        map = map_strip<T, K>(blk.ncols, mask_word);
        total = map.n_slots * K;
        slots = reinterpret_cast<unsigned short*>(strip + slot_table_at);
        write_slot_table(slots, mask_word, map);
    }
    int* const hot_rows = strip + total;
    float worst = 0.f;   // magnitudes of the cut rows on their way into and out of LDS
    if constexpr (!EXACT) {
        // read past the L1 (the row was last written by another compute unit's plain stores)
        for (int slot = wave; slot < n_hot; slot += n_waves) {
            const Row<VEC> p = load_row<VEC, true>(P + (int64_t)uniform_lane(hot_u, slot) * K, lane, active);
#pragma unroll
            for (int j = 0; j < VEC; ++j)
                if (active) hot_rows[slot * K + strip_elem<T>(lane, j)] = to_strip<EXACT>(p.x[j], worst);
        }
    }
    if (copy_in) strip_copy_in<T, K, EXACT, COHERENT, SPARSE>(strip, Qt, blk.col0, blk.ncols, watch, map);
    __syncthreads();

    const float shrink = lr * lambda;
    for (int e = wave; e < blk.n_entries; e += n_waves) {
        if (e != wave) {
            fetch_entry(e);
            if (EXACT || raw_len > 0)
                first_rows = request_first_rows<T, K, DEPTH>(P, mu, min(kWave, raw_len & ~kSharedRowFlag),
                                                                         lane, active);
        }
        const int32_t len = raw_len & ~kSharedRowFlag;
        if constexpr (EXACT) {
            lds_owned_chunk<T, K, DEPTH, true, SPARSE>(P, strip, blk.col0, slots, U, V, R, begin, len, mu, mv, mr,
                                                       first_rows, lr, shrink, lane, active);
        } else {
            if (raw_len < 0) {
                // a piece of a cut row at the front and / or at the back, whole rows between them
                // (the work lists never cut more rows of a block than it has slots in LDS)
                auto slot_of = [&](int u) {
                    const unsigned long long hit = __ballot(hot_u == u);
                    return hit ? (int)__builtin_ctzll(hit) : -1;
                };
                const int u_front = uniform_lane(mu, 0);
                const int u_back = len <= kWave ? uniform_lane(mu, len - 1) : (int)U[begin + len - 1];
                const int front_slot = slot_of(u_front), back_slot = slot_of(u_back);
                const int32_t front = front_slot >= 0 ? run_of_row<false>(U, begin, len, u_front, lane) : 0;
                const int32_t back = back_slot >= 0 && front < len
                                         ? run_of_row<true>(U, begin + front, len - front, u_back, lane) : 0;
                const int32_t between = len - front - back;
                if (between > 0) {
                    // requested now, used after the two pieces
                    if (front > 0 && lane < min(kWave, between)) {
                        mu = U[begin + front + lane];
                        mv = V[begin + front + lane];
                        mr = R[begin + front + lane];
                    }
                    first_rows = request_first_rows<T, K, DEPTH>(P, mu, min(kWave, between), lane, active);
                }
                if (front > 0)
                    lds_hot_row_piece<T, K, SPARSE>(hot_rows + front_slot * K, strip, blk.col0, slots, V, R, begin, front,
                                                    lr, shrink, lane, active, watch);
                if (back > 0)
                    lds_hot_row_piece<T, K, SPARSE>(hot_rows + back_slot * K, strip, blk.col0, slots, V, R,
                                                    begin + len - back, back, lr, shrink, lane, active, watch);
                if (between > 0)
                    lds_hog_chunk<T, K, DEPTH, SPARSE>(P, strip, blk.col0, slots, U, V, R, begin + front, between, mu, mv,
                                                       mr, first_rows, lr, shrink, lane, active, watch);
            } else {
                lds_hog_chunk<T, K, DEPTH, SPARSE>(P, strip, blk.col0, slots, U, V, R, begin, len, mu, mv, mr,
                                                   first_rows, lr, shrink, lane, active, watch);
            }
        }
    }
    __syncthreads();

    if constexpr (!EXACT) {
        for (int slot = wave; slot < n_hot; slot += n_waves) {
            Row<VEC> p;
#pragma unroll
            for (int j = 0; j < VEC; ++j)
                p.x[j] = active ? quantise<T>(from_strip<EXACT>(hot_rows[slot * K + strip_elem<T>(lane, j)], worst)) : 0.f;
            store_row<VEC>(P + (int64_t)uniform_lane(hot_u, slot) * K, lane, active, p);
        }
        watch.see_plain(worst);
    }
    if (copy_out) strip_copy_out<T, K, EXACT, COHERENT, SPARSE>(strip, Qt, blk.col0, blk.ncols, watch, map);
    return true;
}

// One launch per stratum: workgroup i works on the i-th non-empty block of the stratum.
template <typename T, int K, bool EXACT, int DEPTH, bool SPARSE>
__global__ __launch_bounds__(EXACT ? kWave : 1024) void sgd_block_lds(
    T* __restrict__ P, T* __restrict__ Qt, const int32_t* __restrict__ U,
    const int32_t* __restrict__ V, const float* __restrict__ R,
    const int64_t* __restrict__ entry_begin, const int32_t* __restrict__ entry_len, const int64_t* __restrict__ hot_pos,
    const LdsBlock* __restrict__ blocks, float lr, float lambda, int* range_flag, const unsigned* __restrict__ touched,
    int touched_words, int slot_table_at)
{
    extern __shared__ int strip[];            // ncols * K values (fixed point, or fp32 bits if EXACT)
    RangeWatch watch;
    const LdsBlock blk = blocks[blockIdx.x];
    unsigned mask_word = 0xffffffffu;
    if constexpr (SPARSE) {
        const int lane = threadIdx.x & (kWave - 1);
        mask_word = lane < touched_words ? touched[(int64_t)blk.id * touched_words + lane] : 0u;
    }
    lds_block_body<T, K, EXACT, false, DEPTH, SPARSE>(strip, P, Qt, U, V, R, entry_begin, entry_len, hot_pos, blk, lr,
                                                      lambda, true, true, mask_word, slot_table_at, watch,
                                                      [] { return true; });
    if constexpr (!EXACT) {
        if (__any(watch.hit()) && (threadIdx.x & (kWave - 1)) == 0) *range_flag = 1;
    }
}

// One launch per EPOCH: workgroup a keeps block row a for the whole epoch (its rows of P are
// never touched by anyone else) and walks the strata on blocks (a, (a+s) mod grid_c); the column
// strips of Qt rotate through the workgroups (the rotation of distributed SGD, here between
// compute units instead of machines).  `done[a]` counts the steps block row a has finished since
// mf_load_blocks (`first` = its value before this epoch).  Before it reads the strip of step t a
// workgroup makes sure that the most recent earlier user of that strip has reported its step; that
// one waited for its own predecessor (every workgroup waits also when its block is empty), so the
// chain of guarantees is unbroken.
//   Strata in natural order (order == nullptr): the only other user of strip (a+s) mod grid_c
//   is the next block row one stratum earlier, so workgroup a waits for done[a+1] >= first + s
//   (the last block row waits for block row 0 having finished stratum s - (grid_c - grid_r) - 1).
//   Strata in a given order (order[t] = stratum of step t, pos = its inverse): the earlier users
//   of strip c are the block rows a' != a at the steps pos[(c - a') mod grid_c] that lie before
//   t; the first wavefront takes the latest of them (one look-up per block row, a wave-wide
//   maximum) and waits for that block row to have finished that step.
// All grid_r workgroups must be resident at once (checked by the host before launching).
// Every wait is bounded: after spin_limit polls a workgroup raises flags[0] and leaves, and every
// waiting workgroup leaves as soon as it sees the flag, so the grid always drains.  flags[1] is
// the range flag of the fixed-point strip (see RangeWatch).
//
// A step is: request the block's first ratings and rows of P, wait for the strip, strip in, block,
// strip out, wait for the stores' acknowledgement, report.
template <typename T, int K, bool EXACT, int DEPTH, bool SPARSE>
__global__ __launch_bounds__(EXACT ? kWave : 1024) void sgd_ring_lds(
    T* __restrict__ P, T* __restrict__ Qt, const int32_t* __restrict__ U,
    const int32_t* __restrict__ V, const float* __restrict__ R,
    const int64_t* __restrict__ entry_begin, const int32_t* __restrict__ entry_len, const int64_t* __restrict__ hot_pos,
    const LdsBlock* __restrict__ ring_blocks, int grid_r, int grid_c, float lr, float lambda,
    int* done, int first, int* flags, long long spin_limit, const int32_t* __restrict__ order,
    const int32_t* __restrict__ pos, const unsigned* __restrict__ touched, int touched_words, int slot_table_at,
    int n_steps)
{
    extern __shared__ int strip[];
    __shared__ int go;
    const int a = (int)blockIdx.x;
    const int next_row = a + 1 < grid_r ? a + 1 : 0;
    const int lag = a + 1 < grid_r ? 0 : grid_c - grid_r;
    RangeWatch watch;
    // n_steps = grid_c for one epoch; a multiple of it (strata in natural order only) for several
    // epochs in one launch: step t of the launch is stratum t mod grid_c, and the waits below hold
    // across the epochs' boundaries as they do inside an epoch
    for (int t = 0; t < n_steps; ++t) {
        const int s = order ? order[t] : t % grid_c;
        // wait (bounded) until the previous user of this step's column strip has reported it
        // finished; returns false when the workgroup has to leave
        auto wait_for_strip = [&]() -> bool {
            if (threadIdx.x < kWave) {
                int waits_on = next_row;
                int need = first + t - lag;          // value of done[waits_on] to wait for
                bool must_wait = t - lag > 0;
                if (order) {
                    int c = a + s;
                    if (c >= grid_c) c -= grid_c;
                    int latest = -1;                 // latest earlier step at which another block row used strip c
                    for (int other = (int)threadIdx.x; other < grid_r; other += kWave) {
                        int s_other = c - other;
                        if (s_other < 0) s_other += grid_c;
                        const int t_other = pos[s_other];
                        if (other != a && t_other < t) latest = max(latest, t_other);
                    }
#pragma unroll
                    for (int d = 32; d >= 1; d >>= 1) latest = max(latest, __shfl_xor(latest, d, kWave));
                    must_wait = latest >= 0;
                    if (must_wait) {
                        waits_on = c - order[latest];
                        if (waits_on < 0) waits_on += grid_c;
                        need = first + latest + 1;
                    }
                }
                if (threadIdx.x == 0) {
                    int ok = 1;
                    if (must_wait) {
                        long long polls = 0;
                        while (__hip_atomic_load(done + waits_on, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < need) {
                            // every poll is a round trip to memory: the abort flag is looked at on
                            // every 16th only, so that the counter is read twice as often
                            if ((polls & 15) == 15 &&
                                __hip_atomic_load(flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                                ok = 0;
                                break;
                            }
                            if (++polls > spin_limit) {
                                __hip_atomic_store(flags, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                ok = 0;
                                break;
                            }
                            __builtin_amdgcn_s_sleep(2);
                        }
                    }
                    go = ok;
                }
            }
            __syncthreads();
            return go != 0;                        // the same answer in every thread of the workgroup
        };
        const LdsBlock blk = ring_blocks[(int64_t)s * grid_r + a];
        // the block's table of touched columns, one bit word per lane (requested before the wait)
        unsigned mask_word = 0xffffffffu;
        if constexpr (SPARSE) {
            const int lane = threadIdx.x & (kWave - 1);
            mask_word = lane < touched_words ? touched[(int64_t)blk.id * touched_words + lane] : 0u;
        }
        bool ok;
        if (blk.n_entries > 0)
            ok = lds_block_body<T, K, EXACT, true, DEPTH, SPARSE>(strip, P, Qt, U, V, R, entry_begin, entry_len, hot_pos,
                                                                  blk, lr, lambda, true, true, mask_word, slot_table_at,
                                                                  watch, wait_for_strip);
        else
            ok = wait_for_strip();   // an empty block still waits: it passes the guarantee on
        if (!ok) return;
        // every thread's stores of the strip have been acknowledged before the step is
        // reported finished
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0)
            __hip_atomic_store(done + a, first + t + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if constexpr (!EXACT) {
        if (__any(watch.hit()) && (threadIdx.x & (kWave - 1)) == 0) flags[1] = 1;
    }
}

// ------------------------------------------------------------------------------------- RMSE
__device__ __forceinline__ double wave_sum_f64(double x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, kWave);
    return x;
}

// Each wavefront walks batches of 64 entries (grid-stride) and adds (r - p.q)^2 in double;
// one partial per wavefront, written unconditionally so the buffer needs no clearing.
template <typename T, int K>
__global__ __launch_bounds__(kGroupThreads) void rmse_partial(
    const T* __restrict__ P, const T* __restrict__ Qt, const int32_t* __restrict__ U,
    const int32_t* __restrict__ V, const float* __restrict__ R, int64_t count,
    double* __restrict__ partials)
{
    constexpr int VEC = RowShape<T, K>::VEC;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t wave_id = (int64_t)blockIdx.x * kWavesPerGroup + wave;
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerGroup;
    const bool active = lane < RowShape<T, K>::ACTIVE;
    double acc = 0.0;
    for (int64_t base = wave_id * kWave; base < count; base += n_waves * kWave) {
        const int cnt = (int)min((int64_t)kWave, count - base);
        int mu = 0, mv = 0;
        float mr = 0.f;
        if (lane < cnt) {
            mu = U[base + lane];
            mv = V[base + lane];
            mr = R[base + lane];
        }
        for (int i = 0; i < cnt; ++i) {
            const int u = uniform_lane(mu, i);
            const int v = uniform_lane(mv, i);
            const float r = __int_as_float(uniform_lane(__float_as_int(mr), i));
            Row<VEC> p = load_row<VEC, false>(P + (int64_t)u * K, lane, active);
            Row<VEC> q = load_row<VEC, false>(Qt + (int64_t)v * K, lane, active);
            double part = 0.0;
#pragma unroll
            for (int j = 0; j < VEC; ++j) part = fma((double)p.x[j], (double)q.x[j], part);
            const double d = (double)r - wave_sum_f64(part);
            acc = fma(d, d, acc);
        }
    }
    if (lane == 0) partials[wave_id] = acc;
}

// Fixed-order sum of the partials by one workgroup.  count > 0: the result is the root of the mean,
// sqrt(sum / count); count == 0: the sum itself.
__global__ __launch_bounds__(kGroupThreads) void rmse_final(const double* __restrict__ partials,
                                                            int n, int64_t count, double* __restrict__ out)
{
    __shared__ double buf[kGroupThreads];
    double acc = 0.0;
    for (int i = threadIdx.x; i < n; i += kGroupThreads) acc += partials[i];
    buf[threadIdx.x] = acc;
    __syncthreads();
    for (int s = kGroupThreads / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) buf[threadIdx.x] += buf[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = count > 0 ? sqrt(buf[0] / (double)count) : buf[0];
}

// ------------------------------------------------------------------------------------- init
// SplitMix64 output function (published algorithm) as the counter-based mixer.
__device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

template <typename T>
__global__ __launch_bounds__(kGroupThreads) void init_fill(T* __restrict__ X, int64_t count,
                                                           uint64_t key, float scale)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
        const uint64_t h = mix64(key + (uint64_t)i);
        const float u01 = (float)(uint32_t)(h >> 40) * (1.0f / 16777216.0f);
        const float val = u01 * scale;
        if constexpr (sizeof(T) == 2) X[i] = round_to_half(val);
        else X[i] = val;
    }
}

// Table of touched columns: for every block of the list, bit c of its `words` bit words is set
// when the block has a rating in column col0 + c of its strip.  One workgroup per block.  The list
// is made for this kernel: first_entry = the block's first packed position, n_entries = its number
// of ratings (not work-list entries).  totals[0] += touched columns of the block, totals[1] +=
// columns of its strip, totals[2] = the most touched columns of any block.
__global__ __launch_bounds__(kGroupThreads) void mark_touched(const LdsBlock* __restrict__ blocks, int64_t n_blocks,
                                                              const int32_t* __restrict__ V, uint32_t* __restrict__ touched,
                                                              int words, unsigned long long* totals)
{
    __shared__ unsigned bits[kMaxTouchedWords];
    // a workgroup takes every gridDim.x-th block of the list (a grid may have billions of blocks)
    for (int64_t at = blockIdx.x; at < n_blocks; at += gridDim.x) {
        const LdsBlock blk = blocks[at];
        if ((int)threadIdx.x < kMaxTouchedWords) bits[threadIdx.x] = 0u;
        __syncthreads();
        const int64_t begin = blk.first_entry, end = begin + blk.n_entries;
        for (int64_t i = begin + (int64_t)threadIdx.x; i < end; i += (int64_t)blockDim.x) {
            const int c = V[i] - blk.col0;
            if (c >= 0 && c < 32 * words) atomicOr(&bits[c >> 5], 1u << (c & 31));
        }
        __syncthreads();
        if ((int)threadIdx.x < words) touched[(int64_t)blk.id * words + threadIdx.x] = bits[threadIdx.x];
        if (threadIdx.x < kWave) {
            int set = (int)threadIdx.x < words ? __popc(bits[threadIdx.x]) : 0;   // words <= 64 = one wavefront
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) set += __shfl_xor(set, d, kWave);
            if (threadIdx.x == 0) {
                atomicAdd(&totals[0], (unsigned long long)set);
                atomicAdd(&totals[1], (unsigned long long)blk.ncols);
                atomicMax(&totals[2], (unsigned long long)set);
            }
        }
        __syncthreads();   // before the bits are cleared for the next block
    }
}

__global__ void fill_i32(int32_t* out, int64_t count, int32_t value)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) out[i] = value;
}

__global__ void xcc_probe(int32_t* out)
{
    // hardware register XCC_ID (id 20), bits [3:0] = index of the accelerator die
    const unsigned id = __builtin_amdgcn_s_getreg(20 | (0 << 6) | ((4 - 1) << 11));
    if (threadIdx.x == 0) out[blockIdx.x] = (int32_t)(id & 0xf);
}

template <typename T, int K>
hipError_t launch_sgd_t(bool hogwild, void* P, void* Qt, const int32_t* U, const int32_t* V,
                        const float* R, const int64_t* eb, const int32_t* el, int64_t first,
                        int64_t n_entries, float lr, float lambda, hipStream_t stream)
{
    // a launch holds fewer than 2^32 threads: a longer work list goes in slices, in order
    constexpr int64_t kMaxGroups = (int64_t)1 << 22;
    for (int64_t done = 0; done < n_entries; done += kMaxGroups * kWavesPerGroup) {
        const unsigned groups = (unsigned)std::min<int64_t>((n_entries - done) / kWavesPerGroup, kMaxGroups);
        if (hogwild)
            hipLaunchKernelGGL((sgd_chunks<T, K, true>), dim3(groups), dim3(kGroupThreads), 0, stream, (T*)P,
                               (T*)Qt, U, V, R, eb, el, first + done, lr, lambda);
        else
            hipLaunchKernelGGL((sgd_chunks<T, K, false>), dim3(groups), dim3(kGroupThreads), 0, stream, (T*)P,
                               (T*)Qt, U, V, R, eb, el, first + done, lr, lambda);
    }
    return hipGetLastError();
}

template <typename T, int K, bool EXACT, int DEPTH, bool SPARSE>
hipError_t launch_sgd_lds_impl(int waves, void* P, void* Qt, const int32_t* U, const int32_t* V,
                            const float* R, const int64_t* eb, const int32_t* el, const int64_t* hot,
                            const LdsBlock* blocks, int64_t n_blocks, size_t lds_bytes, float lr,
                            float lambda, int* range_flag, const uint32_t* touched, int touched_words,
                            int slot_table_at, hipStream_t stream)
{
    // more than 64 KiB of dynamic LDS has to be allowed once per kernel and device
    static bool raised[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !raised[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sgd_block_lds<T, K, EXACT, DEPTH, SPARSE>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
        if (e != hipSuccess) return e;
        raised[dev] = true;
    }
    hipLaunchKernelGGL((sgd_block_lds<T, K, EXACT, DEPTH, SPARSE>), dim3((unsigned)n_blocks), dim3(waves * kWave), lds_bytes,
                       stream, (T*)P, (T*)Qt, U, V, R, eb, el, hot, blocks, lr, lambda, range_flag, touched, touched_words,
                       slot_table_at);
    return hipGetLastError();
}

template <typename T, int K, bool EXACT, int DEPTH, bool SPARSE>
hipError_t launch_sgd_ring_impl(int waves, bool query_only, int* max_resident, void* P, void* Qt,
                                const int32_t* U, const int32_t* V, const float* R, const int64_t* eb,
                                const int32_t* el, const int64_t* hot, const LdsBlock* ring_blocks, int grid_r, int grid_c,
                                size_t lds_bytes, float lr, float lambda, int* done, int first,
                                int* abort_flag, long long spin_limit, const int32_t* order, const int32_t* pos,
                                const uint32_t* touched, int touched_words, int slot_table_at, int n_steps,
                                hipStream_t stream)
{
    static bool raised[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !raised[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sgd_ring_lds<T, K, EXACT, DEPTH, SPARSE>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
        if (e != hipSuccess) return e;
        raised[dev] = true;
    }
    if (query_only) {
        int per_cu = 0, cus = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, sgd_ring_lds<T, K, EXACT, DEPTH, SPARSE>, waves * kWave,
                                                         lds_bytes);
        if (e != hipSuccess) return e;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        *max_resident = per_cu * cus;
        return hipSuccess;
    }
    hipLaunchKernelGGL((sgd_ring_lds<T, K, EXACT, DEPTH, SPARSE>), dim3((unsigned)grid_r), dim3(waves * kWave), lds_bytes,
                       stream, (T*)P, (T*)Qt, U, V, R, eb, el, hot, ring_blocks, grid_r, grid_c, lr, lambda, done,
                       first, abort_flag, spin_limit, order, pos, touched, touched_words, slot_table_at, n_steps);
    return hipGetLastError();
}

template <typename T, int K>
hipError_t launch_sgd_ring_t(bool exact, bool short_prefetch, int waves, bool query_only, int* max_resident, void* P, void* Qt,
                             const int32_t* U, const int32_t* V, const float* R, const int64_t* eb,
                             const int32_t* el, const int64_t* hot, const LdsBlock* ring_blocks, int grid_r, int grid_c,
                             size_t lds_bytes, float lr, float lambda, int* done, int first, int* abort_flag,
                             long long spin_limit, const int32_t* order, const int32_t* pos, const uint32_t* touched,
                             int touched_words, int slot_table_at, int n_steps, hipStream_t stream)
{
    if (exact && touched)
        return launch_sgd_ring_impl<T, K, true, kDetPrefetchDepth, true>(
            1, query_only, max_resident, P, Qt, U, V, R, eb, el, hot, ring_blocks, grid_r, grid_c, lds_bytes, lr, lambda, done,
            first, abort_flag, spin_limit, order, pos, touched, touched_words, slot_table_at, n_steps, stream);
    if (exact)
        return launch_sgd_ring_impl<T, K, true, kDetPrefetchDepth, false>(
            1, query_only, max_resident, P, Qt, U, V, R, eb, el, hot, ring_blocks, grid_r, grid_c, lds_bytes, lr, lambda, done,
            first, abort_flag, spin_limit, order, pos, nullptr, 0, 0, n_steps, stream);
    // the form that keeps only the touched columns of a strip in LDS exists where a wavefront's piece of
    // the strip lies in one column
    if constexpr (SparseStrip<T, K>::kPossible) {
        if (touched && short_prefetch)
            return launch_sgd_ring_impl<T, K, false, kShortPrefetchDepth, true>(
                waves, query_only, max_resident, P, Qt, U, V, R, eb, el, hot, ring_blocks, grid_r, grid_c, lds_bytes, lr, lambda,
                done, first, abort_flag, spin_limit, order, pos, touched, touched_words, slot_table_at, n_steps, stream);
        if (touched)
            return launch_sgd_ring_impl<T, K, false, kLongPrefetchDepth<T>, true>(
                waves, query_only, max_resident, P, Qt, U, V, R, eb, el, hot, ring_blocks, grid_r, grid_c, lds_bytes, lr, lambda,
                done, first, abort_flag, spin_limit, order, pos, touched, touched_words, slot_table_at, n_steps, stream);
    }
    if (short_prefetch)
        return launch_sgd_ring_impl<T, K, false, kShortPrefetchDepth, false>(
            waves, query_only, max_resident, P, Qt, U, V, R, eb, el, hot, ring_blocks, grid_r, grid_c, lds_bytes, lr, lambda, done,
            first, abort_flag, spin_limit, order, pos, nullptr, 0, 0, n_steps, stream);
    return launch_sgd_ring_impl<T, K, false, kLongPrefetchDepth<T>, false>(
        waves, query_only, max_resident, P, Qt, U, V, R, eb, el, hot, ring_blocks, grid_r, grid_c, lds_bytes, lr, lambda, done,
        first, abort_flag, spin_limit, order, pos, nullptr, 0, 0, n_steps, stream);
}

template <typename T, int K>
hipError_t launch_sgd_lds_t(bool exact, bool short_prefetch, int waves, void* P, void* Qt, const int32_t* U, const int32_t* V,
                            const float* R, const int64_t* eb, const int32_t* el, const int64_t* hot,
                            const LdsBlock* blocks, int64_t n_blocks, size_t lds_bytes, float lr,
                            float lambda, int* range_flag, const uint32_t* touched, int touched_words, int slot_table_at,
                            hipStream_t stream)
{
    if (exact && touched)
        return launch_sgd_lds_impl<T, K, true, kDetPrefetchDepth, true>(1, P, Qt, U, V, R, eb, el, hot, blocks, n_blocks,
                                                                        lds_bytes, lr, lambda, range_flag, touched,
                                                                        touched_words, slot_table_at, stream);
    if (exact)
        return launch_sgd_lds_impl<T, K, true, kDetPrefetchDepth, false>(1, P, Qt, U, V, R, eb, el, hot, blocks, n_blocks,
                                                                         lds_bytes, lr, lambda, range_flag, nullptr, 0, 0,
                                                                         stream);
    if constexpr (SparseStrip<T, K>::kPossible) {
        if (touched && short_prefetch)
            return launch_sgd_lds_impl<T, K, false, kShortPrefetchDepth, true>(
                waves, P, Qt, U, V, R, eb, el, hot, blocks, n_blocks, lds_bytes, lr, lambda, range_flag, touched,
                touched_words, slot_table_at, stream);
        if (touched)
            return launch_sgd_lds_impl<T, K, false, kLongPrefetchDepth<T>, true>(
                waves, P, Qt, U, V, R, eb, el, hot, blocks, n_blocks, lds_bytes, lr, lambda, range_flag, touched,
                touched_words, slot_table_at, stream);
    }
    if (short_prefetch)
        return launch_sgd_lds_impl<T, K, false, kShortPrefetchDepth, false>(waves, P, Qt, U, V, R, eb, el, hot, blocks,
                                                                            n_blocks, lds_bytes, lr, lambda, range_flag,
                                                                            nullptr, 0, 0, stream);
    return launch_sgd_lds_impl<T, K, false, kLongPrefetchDepth<T>, false>(waves, P, Qt, U, V, R, eb, el, hot, blocks, n_blocks,
                                                                      lds_bytes, lr, lambda, range_flag, nullptr, 0, 0,
                                                                      stream);
}

template <typename T, int K>
hipError_t launch_rmse_t(const void* P, const void* Qt, const int32_t* U, const int32_t* V,
                         const float* R, int64_t count, double* partials, double* sum_out, bool root,
                         hipStream_t stream)
{
    hipLaunchKernelGGL((rmse_partial<T, K>), dim3(kRmseGroups), dim3(kGroupThreads), 0, stream,
                       (const T*)P, (const T*)Qt, U, V, R, count, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rmse_final, dim3(1), dim3(kGroupThreads), 0, stream, partials, kRmsePartials,
                       root ? count : (int64_t)0, sum_out);
    return hipGetLastError();
}

}  // namespace

#define MF_DISPATCH(FN, ...)                                                     \
    do {                                                                         \
        if (dtype == MF_F32) {                                                   \
            switch (k) {                                                         \
                case 32: return FN<float, 32>(__VA_ARGS__);                      \
                case 64: return FN<float, 64>(__VA_ARGS__);                      \
                case 128: return FN<float, 128>(__VA_ARGS__);                    \
                case 256: return FN<float, 256>(__VA_ARGS__);                    \
            }                                                                    \
        } else if (dtype == MF_F16) {                                            \
            switch (k) {                                                         \
                case 32: return FN<__half, 32>(__VA_ARGS__);                     \
                case 64: return FN<__half, 64>(__VA_ARGS__);                     \
                case 128: return FN<__half, 128>(__VA_ARGS__);                   \
                case 256: return FN<__half, 256>(__VA_ARGS__);                   \
            }                                                                    \
        }                                                                        \
        return hipErrorInvalidValue;                                             \
    } while (0)

hipError_t launch_sgd(int dtype, int k, bool hogwild, void* P, void* Qt, const int32_t* U,
                      const int32_t* V, const float* R, const int64_t* entry_begin,
                      const int32_t* entry_len, int64_t first_entry, int64_t n_entries, float lr,
                      float lambda, hipStream_t stream)
{
    if (n_entries <= 0) return hipSuccess;
    if (n_entries % kWavesPerGroup) return hipErrorInvalidValue;
    MF_DISPATCH(launch_sgd_t, hogwild, P, Qt, U, V, R, entry_begin, entry_len, first_entry, n_entries, lr,
                lambda, stream);
}

size_t lds_strip_bytes(int k, int32_t max_cols) { return (size_t)max_cols * k * sizeof(float); }

hipError_t launch_sgd_lds(int dtype, int k, bool exact, bool short_prefetch, int waves, void* P, void* Qt, const int32_t* U,
                          const int32_t* V, const float* R, const int64_t* entry_begin,
                          const int32_t* entry_len, const int64_t* hot_pos, const LdsBlock* blocks, int64_t n_blocks,
                          size_t lds_bytes, float lr, float lambda, int* range_flag, const uint32_t* touched,
                          int touched_words, int slot_table_at, hipStream_t stream)
{
    if (n_blocks <= 0) return hipSuccess;
    if (waves < 1 || waves > 16 || lds_bytes > kLdsBudget || !range_flag) return hipErrorInvalidValue;
    if (touched && (touched_words < 1 || touched_words > kMaxTouchedWords || slot_table_at < 0 ||
                    (size_t)slot_table_at * 4 + (size_t)touched_words * 64 > lds_bytes))
        return hipErrorInvalidValue;
    MF_DISPATCH(launch_sgd_lds_t, exact, short_prefetch, waves, P, Qt, U, V, R, entry_begin, entry_len, hot_pos, blocks, n_blocks,
                lds_bytes, lr, lambda, range_flag, touched, touched_words, slot_table_at, stream);
}

hipError_t launch_sgd_ring(int dtype, int k, bool exact, bool short_prefetch, int waves, bool query_only, int* max_resident,
                           void* P, void* Qt, const int32_t* U, const int32_t* V, const float* R,
                           const int64_t* entry_begin, const int32_t* entry_len, const int64_t* hot_pos, const LdsBlock* ring_blocks,
                           int grid_r, int grid_c, size_t lds_bytes, float lr, float lambda, int* done,
                           int first, int* abort_flag, long long spin_limit, const int32_t* order,
                           const int32_t* pos, const uint32_t* touched, int touched_words, int slot_table_at,
                           int n_epochs, hipStream_t stream)
{
    if (waves < 1 || waves > 16 || lds_bytes > kLdsBudget || grid_r < 1) return hipErrorInvalidValue;
    if (n_epochs < 1 || (order && n_epochs != 1) || (int64_t)n_epochs * grid_c > ((int64_t)1 << 30)) return hipErrorInvalidValue;
    const int n_steps = n_epochs * grid_c;
    if ((order == nullptr) != (pos == nullptr)) return hipErrorInvalidValue;
    if (touched && (touched_words < 1 || touched_words > kMaxTouchedWords || slot_table_at < 0 ||
                    (size_t)slot_table_at * 4 + (size_t)touched_words * 64 > lds_bytes))
        return hipErrorInvalidValue;
    MF_DISPATCH(launch_sgd_ring_t, exact, short_prefetch, waves, query_only, max_resident, P, Qt, U, V, R, entry_begin,
                entry_len, hot_pos, ring_blocks, grid_r, grid_c, lds_bytes, lr, lambda, done, first, abort_flag,
                spin_limit, order, pos, touched, touched_words, slot_table_at, n_steps, stream);
}

hipError_t launch_mark_touched(const LdsBlock* blocks, int64_t n_blocks, const int32_t* V, uint32_t* touched, int words,
                               unsigned long long* totals, hipStream_t stream)
{
    if (n_blocks <= 0) return hipSuccess;
    if (words < 1 || words > kMaxTouchedWords) return hipErrorInvalidValue;
    // a launch holds fewer than 2^32 threads in a dimension: workgroups loop over the list
    const unsigned groups = (unsigned)std::min<int64_t>(n_blocks, (int64_t)1 << 20);
    hipLaunchKernelGGL(mark_touched, dim3(groups), dim3(kGroupThreads), 0, stream, blocks, n_blocks, V, touched, words,
                       totals);
    return hipGetLastError();
}

hipError_t launch_rmse(int dtype, int k, const void* P, const void* Qt, const int32_t* U,
                       const int32_t* V, const float* R, int64_t count, double* partials,
                       double* sum_out, bool root, hipStream_t stream)
{
    MF_DISPATCH(launch_rmse_t, P, Qt, U, V, R, count, partials, sum_out, root, stream);
}

hipError_t launch_init(int dtype, void* X, int64_t count, uint64_t seed, uint64_t stream_id,
                       float scale, hipStream_t stream)
{
    if (count <= 0) return hipSuccess;
    uint64_t z = seed ^ (stream_id * 0xD1B54A32D192ED03ULL);
    // same mixer as on the device, evaluated once on the host for the stream key
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    const uint64_t key = z ^ (z >> 31);
    const unsigned groups = (unsigned)std::min<int64_t>((count + kGroupThreads - 1) / kGroupThreads, 8192);
    if (dtype == MF_F32)
        hipLaunchKernelGGL(init_fill<float>, dim3(groups), dim3(kGroupThreads), 0, stream, (float*)X, count, key, scale);
    else if (dtype == MF_F16)
        hipLaunchKernelGGL(init_fill<__half>, dim3(groups), dim3(kGroupThreads), 0, stream, (__half*)X, count, key, scale);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_fill_i32(int32_t* d_out, int64_t count, int32_t value, hipStream_t stream)
{
    if (count <= 0) return hipSuccess;
    const int64_t groups = std::min<int64_t>((count + kGroupThreads - 1) / kGroupThreads, (int64_t)1 << 20);
    hipLaunchKernelGGL(fill_i32, dim3((unsigned)groups), dim3(kGroupThreads), 0, stream, d_out, count, value);
    return hipGetLastError();
}

hipError_t launch_xcc_probe(int32_t n_groups, int32_t* d_out, hipStream_t stream)
{
    hipLaunchKernelGGL(xcc_probe, dim3((unsigned)n_groups), dim3(kWave), 0, stream, d_out);
    return hipGetLastError();
}

}  // namespace mf
