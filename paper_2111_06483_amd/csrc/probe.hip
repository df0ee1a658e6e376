// Bandwidth probes: plain kernels that measure, on the machine at hand, the
// ceilings the aggregation kernels are compared with -- a streaming read, a
// copy, and random gathers of whole feature rows with the access shape of the
// aggregation kernels (one wavefront per row, 16 bytes per lane, 8 rows in
// flight) but no arithmetic to speak of.
//
// Measurement tooling, not part of the method: built into its own shared object
// (libsar_bench.so, header include/sar_bench_probes.h) that only bench.py loads.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <type_traits>

#include "../../include/sar_bench_probes.h"

namespace {

constexpr int kProbeWGs = 256 * 8;   // 256 CUs x 8 resident workgroups

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline int launched() { return hipGetLastError() == hipSuccess ? 0 : -3; }

__global__ __launch_bounds__(256) void k_probe_read(const float4* __restrict__ p, size_t n4, int reps,
                                                    float* __restrict__ sink)
{
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    const size_t stride = (size_t)gridDim.x * 256;
    for (int r = 0; r < reps; ++r)
        for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
            const float4 v = p[i];
            a.x += v.x;
            a.y += v.y;
            a.z += v.z;
            a.w += v.w;
        }
    if (a.x + a.y + a.z + a.w == 1.2345e38f) sink[0] = 1.f;   // keeps the loads alive
}

__global__ __launch_bounds__(256) void k_probe_copy(const float4* __restrict__ src, float4* __restrict__ dst,
                                                    size_t n4)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) dst[i] = src[i];
}

template <int LANE_BYTES>
__global__ __launch_bounds__(256) void k_probe_gather(const char* __restrict__ rows, int row_bytes,
                                                      const int32_t* __restrict__ idx, int64_t n_idx,
                                                      float* __restrict__ sink)
{
    constexpr int U = 8;
    using V = typename std::conditional<LANE_BYTES == 16, float4, float2>::type;
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * 256) >> 6;
    float acc = 0.f;
    for (int64_t base = wave * U; base + U <= n_idx; base += n_waves * U) {
        V v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int j = __builtin_amdgcn_readfirstlane(idx[base + k]);
            v[k] = *reinterpret_cast<const V*>(rows + (int64_t)j * row_bytes + lane * LANE_BYTES);
        }
#pragma unroll
        for (int k = 0; k < U; ++k) acc += v[k].x + v[k].y;
    }
    if (acc == 1.2345e38f) sink[0] = 1.f;
}

// The same gathers, and after every 8 of them `w` of the gathered rows are written to consecutive
// rows of `out`: the read/write mix of the backward kernels (each source row read and its error
// row written once, a few gathered rows in between) without their arithmetic.
template <int LANE_BYTES>
__global__ __launch_bounds__(256) void k_probe_gather_write(const char* __restrict__ rows, int row_bytes,
                                                            const int32_t* __restrict__ idx, int64_t n_idx, int w,
                                                            char* __restrict__ out)
{
    constexpr int U = 8;
    using V = typename std::conditional<LANE_BYTES == 16, float4, float2>::type;
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * 256) >> 6;
    float acc = 0.f;
    for (int64_t base = wave * U; base + U <= n_idx; base += n_waves * U) {
        V v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int j = __builtin_amdgcn_readfirstlane(idx[base + k]);
            v[k] = *reinterpret_cast<const V*>(rows + (int64_t)j * row_bytes + lane * LANE_BYTES);
        }
        const int64_t o = base / U * w;
#pragma unroll
        for (int k = 0; k < U; ++k) {
            acc += v[k].x + v[k].y;     // every gathered row is used, written or not
            if (k < w) *reinterpret_cast<V*>(out + (o + k) * row_bytes + lane * LANE_BYTES) = v[k];
        }
    }
    if (acc == 1.2345e38f) out[0] = 1;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" int sar_bench_stream_read(const void* buf, size_t bytes, int reps, float* sink, void* stream)
{
    if (!(buf && sink && aligned16(buf))) return -1;
    if (!(reps >= 1)) return -1;
    k_probe_read<<<kProbeWGs, 256, 0, as_stream(stream)>>>(static_cast<const float4*>(buf), bytes / 16,
                                                                         reps, sink);
    return launched();
}

extern "C" int sar_bench_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    if (!(src && dst && aligned16(src) && aligned16(dst))) return -1;
    k_probe_copy<<<kProbeWGs, 256, 0, as_stream(stream)>>>(static_cast<const float4*>(src),
                                                                         static_cast<float4*>(dst), bytes / 16);
    return launched();
}

extern "C" int sar_bench_row_gather(const void* rows, int64_t n_rows, int row_bytes, const int32_t* idx,
                                    int64_t n_idx, float* sink, void* stream)
{
    if (!(rows && idx && sink && aligned16(rows))) return -1;
    if (!(n_rows > 0 && n_idx >= 0)) return -1;
    if (row_bytes != 1024 && row_bytes != 512) return -2;
    hipStream_t st = as_stream(stream);
    if (row_bytes == 1024)
        k_probe_gather<16><<<kProbeWGs, 256, 0, st>>>(static_cast<const char*>(rows), row_bytes, idx, n_idx, sink);
    else
        k_probe_gather<8><<<kProbeWGs, 256, 0, st>>>(static_cast<const char*>(rows), row_bytes, idx, n_idx, sink);
    return launched();
}

extern "C" int sar_bench_gather_write(const void* rows, int64_t n_rows, int row_bytes, const int32_t* idx,
                                      int64_t n_idx, int writes_per_8, void* out, void* stream)
{
    if (!(rows && idx && out && aligned16(rows) && aligned16(out))) return -1;
    if (!(n_rows > 0 && n_idx >= 0)) return -1;
    if (!(writes_per_8 >= 0 && writes_per_8 <= 8)) return -1;
    if (row_bytes != 1024 && row_bytes != 512) return -2;
    hipStream_t st = as_stream(stream);
    if (row_bytes == 1024)
        k_probe_gather_write<16><<<kProbeWGs, 256, 0, st>>>(static_cast<const char*>(rows), row_bytes, idx, n_idx,
                                                                    writes_per_8, static_cast<char*>(out));
    else
        k_probe_gather_write<8><<<kProbeWGs, 256, 0, st>>>(static_cast<const char*>(rows), row_bytes, idx, n_idx,
                                                                   writes_per_8, static_cast<char*>(out));
    return launched();
}
