// Device code of libmf_sgd for gfx950 (CDNA4, 64-wide wavefronts).
//
// sgd_chunks   : the training step of the paper's Algorithm 1 -- e = r - p.q, then
//                p += lr*(e*q - lambda*p), q += lr*(e*p - lambda*q) with the old p on the right --
//                one wavefront per work-list entry, one rating at a time, the k factors of a
//                row spread over the lanes, the dot product reduced with DPP cross-lane adds.
// rmse_partial : sum of squared prediction errors (Eq. 1 against the rating), double precision.
// init_fill    : counter-based uniform initial factors.
//
// This is a gather / dot / scatter over rows of 128..1024 bytes: it is bound by memory traffic
// and latency, so there is no MFMA here; the lanes hold rows in registers, consecutive ratings
// of one matrix row reuse p_u from registers, and the next rating's rows are requested before
// the current rating is computed.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "../../include/mf_sgd.h"
#include "mf_internal.h"

namespace mf {
namespace {

// ---------------------------------------------------------------------------------- row access
// A factor row of K elements is held by a wavefront as VEC consecutive elements per lane;
// lanes >= K / VEC (only for K = 32) hold zeros and never touch memory.
template <int K>
struct RowShape {
    static constexpr int VEC = K >= 64 ? K / 64 : 1;
    static constexpr int ACTIVE = K / VEC;
};

template <int VEC>
struct Row {
    float x[VEC];
};

template <int VEC>
__device__ __forceinline__ Row<VEC> load_row(const float* row_ptr, int lane, bool active)
{
    Row<VEC> r;
#pragma unroll
    for (int j = 0; j < VEC; ++j) r.x[j] = 0.f;
    if (active) {
        if constexpr (VEC == 1) {
            r.x[0] = row_ptr[lane];
        } else if constexpr (VEC == 2) {
            float2 t = *reinterpret_cast<const float2*>(row_ptr + 2 * lane);
            r.x[0] = t.x;
            r.x[1] = t.y;
        } else {
            float4 t = *reinterpret_cast<const float4*>(row_ptr + 4 * lane);
            r.x[0] = t.x;
            r.x[1] = t.y;
            r.x[2] = t.z;
            r.x[3] = t.w;
        }
    }
    return r;
}

template <int VEC>
__device__ __forceinline__ Row<VEC> load_row(const __half* row_ptr, int lane, bool active)
{
    Row<VEC> r;
#pragma unroll
    for (int j = 0; j < VEC; ++j) r.x[j] = 0.f;
    if (active) {
        if constexpr (VEC == 1) {
            r.x[0] = __half2float(row_ptr[lane]);
        } else if constexpr (VEC == 2) {
            __half2 t = *reinterpret_cast<const __half2*>(row_ptr + 2 * lane);
            r.x[0] = __low2float(t);
            r.x[1] = __high2float(t);
        } else {
            uint2 raw = *reinterpret_cast<const uint2*>(row_ptr + 4 * lane);
            __half2 a = *reinterpret_cast<__half2*>(&raw.x);
            __half2 b = *reinterpret_cast<__half2*>(&raw.y);
            r.x[0] = __low2float(a);
            r.x[1] = __high2float(a);
            r.x[2] = __low2float(b);
            r.x[3] = __high2float(b);
        }
    }
    return r;
}

template <int VEC>
__device__ __forceinline__ void store_row(float* row_ptr, int lane, bool active, const Row<VEC>& r)
{
    if (!active) return;
    if constexpr (VEC == 1) {
        row_ptr[lane] = r.x[0];
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2*>(row_ptr + 2 * lane) = make_float2(r.x[0], r.x[1]);
    } else {
        *reinterpret_cast<float4*>(row_ptr + 4 * lane) = make_float4(r.x[0], r.x[1], r.x[2], r.x[3]);
    }
}

// binary16 storage: the row kept in registers already holds values on the binary16 grid
// (see quantise), so the conversion below is exact.
template <int VEC>
__device__ __forceinline__ void store_row(__half* row_ptr, int lane, bool active, const Row<VEC>& r)
{
    if (!active) return;
    if constexpr (VEC == 1) {
        row_ptr[lane] = __float2half_rn(r.x[0]);
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<__half2*>(row_ptr + 2 * lane) = __floats2half2_rn(r.x[0], r.x[1]);
    } else {
        __half2 a = __floats2half2_rn(r.x[0], r.x[1]);
        __half2 b = __floats2half2_rn(r.x[2], r.x[3]);
        uint2 raw;
        raw.x = *reinterpret_cast<unsigned*>(&a);
        raw.y = *reinterpret_cast<unsigned*>(&b);
        *reinterpret_cast<uint2*>(row_ptr + 4 * lane) = raw;
    }
}

// Values leave a step on the grid of the storage type: fp32 as they are, binary16 rounded to
// nearest even after EVERY step, also while a row stays in registers across several ratings.
template <typename T>
__device__ __forceinline__ float quantise(float x)
{
    if constexpr (sizeof(T) == 2) return __half2float(__float2half_rn(x));
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
//      the store of rating i-1 and would be stale).
template <typename T, int K>
__global__ __launch_bounds__(kGroupThreads) void sgd_chunks(
    T* __restrict__ P, T* __restrict__ Qt, const int32_t* __restrict__ U,
    const int32_t* __restrict__ V, const float* __restrict__ R,
    const int64_t* __restrict__ entry_begin, const int32_t* __restrict__ entry_len,
    int64_t first_entry, float lr, float lambda)
{
    constexpr int VEC = RowShape<K>::VEC;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t entry = first_entry + (int64_t)blockIdx.x * kWavesPerGroup + wave;
    const int32_t len = entry_len[entry];
    if (len == 0) return;
    const int64_t begin = entry_begin[entry];
    const bool active = lane < RowShape<K>::ACTIVE;
    const float shrink = lr * lambda;

    Row<VEC> p, q;
    int cur_u = -1;
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
            if (cur_u >= 0) store_row<VEC>(P + (int64_t)cur_u * K, lane, active, p);
            p = load_row<VEC>(P + (int64_t)u * K, lane, active);
            cur_u = u;
        }
        q = load_row<VEC>(Qt + (int64_t)v * K, lane, active);
        for (int i = 0; i < cnt; ++i) {
            const float r = __int_as_float(uniform_lane(__float_as_int(mr), i));
            // request the rows of the next rating of this batch before computing this one
            const bool more = i + 1 < cnt;
            int un = u, vn = v;
            Row<VEC> pn, qn;
            if (more) {
                un = uniform_lane(mu, i + 1);
                vn = uniform_lane(mv, i + 1);
                qn = load_row<VEC>(Qt + (int64_t)vn * K, lane, active);
                if (un != u) pn = load_row<VEC>(P + (int64_t)un * K, lane, active);
            }
            float part = 0.f;
#pragma unroll
            for (int j = 0; j < VEC; ++j) part = fmaf(p.x[j], q.x[j], part);
            const float e = r - wave_sum(part);
            const float step = lr * e;
            Row<VEC> p2, q2;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                // p + lr*(e*q - lambda*p) regrouped as (p - (lr*lambda)*p) + (lr*e)*q: two
                // fused operations, each rounded once at the magnitude of the element
                p2.x[j] = quantise<T>(fmaf(step, q.x[j], fmaf(-shrink, p.x[j], p.x[j])));
                q2.x[j] = quantise<T>(fmaf(step, p.x[j], fmaf(-shrink, q.x[j], q.x[j])));
            }
            store_row<VEC>(Qt + (int64_t)v * K, lane, active, q2);
            if (more) {
                if (un != u) {
                    store_row<VEC>(P + (int64_t)u * K, lane, active, p2);
                    p = pn;
                    cur_u = un;
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
    store_row<VEC>(P + (int64_t)cur_u * K, lane, active, p);
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
    constexpr int VEC = RowShape<K>::VEC;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t wave_id = (int64_t)blockIdx.x * kWavesPerGroup + wave;
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerGroup;
    const bool active = lane < RowShape<K>::ACTIVE;
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
            Row<VEC> p = load_row<VEC>(P + (int64_t)u * K, lane, active);
            Row<VEC> q = load_row<VEC>(Qt + (int64_t)v * K, lane, active);
            double part = 0.0;
#pragma unroll
            for (int j = 0; j < VEC; ++j) part = fma((double)p.x[j], (double)q.x[j], part);
            const double d = (double)r - wave_sum_f64(part);
            acc = fma(d, d, acc);
        }
    }
    if (lane == 0) partials[wave_id] = acc;
}

// Fixed-order sum of the partials by one workgroup.
__global__ __launch_bounds__(kGroupThreads) void rmse_final(const double* __restrict__ partials,
                                                            int n, double* __restrict__ out)
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
    if (threadIdx.x == 0) out[0] = buf[0];
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
        if constexpr (sizeof(T) == 2) X[i] = __float2half_rn(val);
        else X[i] = val;
    }
}

__global__ void xcc_probe(int32_t* out)
{
    // hardware register XCC_ID (id 20), bits [3:0] = index of the accelerator die
    const unsigned id = __builtin_amdgcn_s_getreg(20 | (0 << 6) | ((4 - 1) << 11));
    if (threadIdx.x == 0) out[blockIdx.x] = (int32_t)(id & 0xf);
}

template <typename T, int K>
hipError_t launch_sgd_t(void* P, void* Qt, const int32_t* U, const int32_t* V, const float* R,
                        const int64_t* eb, const int32_t* el, int64_t first, int64_t n_entries,
                        float lr, float lambda, hipStream_t stream)
{
    const unsigned groups = (unsigned)(n_entries / kWavesPerGroup);
    hipLaunchKernelGGL((sgd_chunks<T, K>), dim3(groups), dim3(kGroupThreads), 0, stream, (T*)P, (T*)Qt, U,
                       V, R, eb, el, first, lr, lambda);
    return hipGetLastError();
}

template <typename T, int K>
hipError_t launch_rmse_t(const void* P, const void* Qt, const int32_t* U, const int32_t* V,
                         const float* R, int64_t count, double* partials, double* sum_out,
                         hipStream_t stream)
{
    hipLaunchKernelGGL((rmse_partial<T, K>), dim3(kRmseGroups), dim3(kGroupThreads), 0, stream,
                       (const T*)P, (const T*)Qt, U, V, R, count, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rmse_final, dim3(1), dim3(kGroupThreads), 0, stream, partials, kRmsePartials,
                       sum_out);
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

hipError_t launch_sgd(int dtype, int k, void* P, void* Qt, const int32_t* U, const int32_t* V,
                      const float* R, const int64_t* entry_begin, const int32_t* entry_len,
                      int64_t first_entry, int64_t n_entries, float lr, float lambda,
                      hipStream_t stream)
{
    if (n_entries <= 0) return hipSuccess;
    if (n_entries % kWavesPerGroup) return hipErrorInvalidValue;
    MF_DISPATCH(launch_sgd_t, P, Qt, U, V, R, entry_begin, entry_len, first_entry, n_entries, lr,
                lambda, stream);
}

hipError_t launch_rmse(int dtype, int k, const void* P, const void* Qt, const int32_t* U,
                       const int32_t* V, const float* R, int64_t count, double* partials,
                       double* sum_out, hipStream_t stream)
{
    MF_DISPATCH(launch_rmse_t, P, Qt, U, V, R, count, partials, sum_out, stream);
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

hipError_t launch_xcc_probe(int32_t n_groups, int32_t* d_out, hipStream_t stream)
{
    hipLaunchKernelGGL(xcc_probe, dim3((unsigned)n_groups), dim3(kWave), 0, stream, d_out);
    return hipGetLastError();
}

}  // namespace mf
