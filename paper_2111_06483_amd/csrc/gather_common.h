// Device helpers shared by the row-gather kernels (sum/mean aggregation and
// the fused attention kernels).
//
// Mapping used throughout: a feature row of F values is covered by G lanes of
// a 64-wide wavefront, each lane owning VEC consecutive values moved with one
// 16-byte access (4 fp32 or 8 bf16).  G is the power of two >= F/VEC, so a
// 1 KiB fp32 row (F = 256) is one fully coalesced wave-wide load.  When G < 64
// the wavefront is cut into SLOTS = 64/G lane groups that work on different
// edges of the same row and are merged at the end.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sar {

struct bf16_t {
    uint16_t bits;
};

constexpr int kWave = 64;
constexpr int kGatherThreads = 256;          // 4 wavefronts per workgroup
constexpr int kWavesPerWG = kGatherThreads / kWave;
constexpr int kMaxPersistentWGs = 256 * 8;   // 256 CUs x 8 resident workgroups

template <typename T>
struct Vec;

template <>
struct Vec<float> {
    static constexpr int N = 4;
    using Raw = float4;
    static __device__ inline Raw load(const float* p) { return *reinterpret_cast<const float4*>(p); }
    static __device__ inline Raw zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ inline void unpack(const Raw& r, float (&v)[4])
    {
        v[0] = r.x;
        v[1] = r.y;
        v[2] = r.z;
        v[3] = r.w;
    }
    static __device__ inline void store(float* p, const float (&v)[4])
    {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};

// fp32 -> bf16, round to nearest even, by the hardware's own conversion (V_CVT_PK_BF16_F32 takes
// two values per instruction): every bf16 value the library stores goes through these two, so
// a row rounded in one kernel equals the same row rounded in another.
typedef __bf16 hw_bf16x2 __attribute__((ext_vector_type(2)));
typedef float hw_f32x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack2_bf16(float lo, float hi)     // lo in bits 0..15
{
    const hw_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, hw_bf16x2));
}
__device__ inline uint32_t f32_to_bf16_rne(float f) { return pack2_bf16(f, 0.f) & 0xffffu; }

template <>
struct Vec<bf16_t> {
    static constexpr int N = 8;
    using Raw = uint4;
    static __device__ inline Raw load(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
    static __device__ inline Raw zero() { return make_uint4(0u, 0u, 0u, 0u); }
    static __device__ inline void unpack(const Raw& r, float (&v)[8])
    {
        v[0] = __uint_as_float(r.x << 16);
        v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16);
        v[3] = __uint_as_float(r.y & 0xffff0000u);
        v[4] = __uint_as_float(r.z << 16);
        v[5] = __uint_as_float(r.z & 0xffff0000u);
        v[6] = __uint_as_float(r.w << 16);
        v[7] = __uint_as_float(r.w & 0xffff0000u);
    }
    static __device__ inline void store(bf16_t* p, const float (&v)[8])
    {
        uint4 r;
        r.x = pack2_bf16(v[0], v[1]);
        r.y = pack2_bf16(v[2], v[3]);
        r.z = pack2_bf16(v[4], v[5]);
        r.w = pack2_bf16(v[6], v[7]);
        *reinterpret_cast<uint4*>(p) = r;
    }
};

// Narrow row types: the same storage moved in lane pieces of fewer than 16 bytes, for head widths
// (or row widths) that are not a whole number of 16-byte pieces.  sizeof(Piece) is one stored
// value, so pointer arithmetic on a Piece* counts values like it does on float* / bf16_t*.
template <typename Base, int N>
struct Piece {
    Base v;
};
using f32x2_t = Piece<float, 2>;     // fp32 rows, 8 bytes per lane
using f32x1_t = Piece<float, 1>;     //            4 bytes
using bf16x4_t = Piece<bf16_t, 4>;   // bf16 rows, 8 bytes per lane
using bf16x2_t = Piece<bf16_t, 2>;   //            4 bytes
using bf16x1_t = Piece<bf16_t, 1>;   //            2 bytes

template <int NN>
struct Vec<Piece<float, NN>> {
    static constexpr int N = NN;
    static_assert(N == 1 || N == 2, "fp32 pieces of 4 or 8 bytes");
    using T = Piece<float, N>;
    struct Raw {
        float v[N];
    };
    static __device__ inline Raw load(const T* p)
    {
        Raw r;
        if constexpr (N == 2) {
            const float2 x = *reinterpret_cast<const float2*>(p);
            r.v[0] = x.x;
            r.v[1] = x.y;
        } else {
            r.v[0] = *reinterpret_cast<const float*>(p);
        }
        return r;
    }
    static __device__ inline Raw zero()
    {
        Raw r;
#pragma unroll
        for (int k = 0; k < N; ++k) r.v[k] = 0.f;
        return r;
    }
    static __device__ inline void unpack(const Raw& r, float (&v)[N])
    {
#pragma unroll
        for (int k = 0; k < N; ++k) v[k] = r.v[k];
    }
    static __device__ inline void store(T* p, const float (&v)[N])
    {
        if constexpr (N == 2)
            *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
        else
            *reinterpret_cast<float*>(p) = v[0];
    }
};

template <int NN>
struct Vec<Piece<bf16_t, NN>> {
    static constexpr int N = NN;
    static_assert(N == 1 || N == 2 || N == 4, "bf16 pieces of 2, 4 or 8 bytes");
    using T = Piece<bf16_t, N>;
    struct Raw {
        uint32_t w[N == 4 ? 2 : 1];
    };
    static __device__ inline Raw load(const T* p)
    {
        Raw r;
        if constexpr (N == 4) {
            const uint2 x = *reinterpret_cast<const uint2*>(p);
            r.w[0] = x.x;
            r.w[1] = x.y;
        } else if constexpr (N == 2) {
            r.w[0] = *reinterpret_cast<const uint32_t*>(p);
        } else {
            r.w[0] = *reinterpret_cast<const uint16_t*>(p);
        }
        return r;
    }
    static __device__ inline Raw zero()
    {
        Raw r;
        r.w[0] = 0u;
        if constexpr (N == 4) r.w[1] = 0u;
        return r;
    }
    static __device__ inline void unpack(const Raw& r, float (&v)[N])
    {
        if constexpr (N == 1) {
            v[0] = __uint_as_float(r.w[0] << 16);
        } else {
#pragma unroll
            for (int k = 0; k < N / 2; ++k) {
                v[2 * k] = __uint_as_float(r.w[k] << 16);
                v[2 * k + 1] = __uint_as_float(r.w[k] & 0xffff0000u);
            }
        }
    }
    static __device__ inline void store(T* p, const float (&v)[N])
    {
        if constexpr (N == 1) {
            *reinterpret_cast<uint16_t*>(p) = (uint16_t)f32_to_bf16_rne(v[0]);
        } else if constexpr (N == 2) {
            *reinterpret_cast<uint32_t*>(p) = pack2_bf16(v[0], v[1]);
        } else {
            *reinterpret_cast<uint2*>(p) = make_uint2(pack2_bf16(v[0], v[1]),
                                                      pack2_bf16(v[2], v[3]));
        }
    }
};

// fp32 rows of N values (the accumulator rows): 16 bytes at a time, or one narrower access
template <int N>
__device__ inline void load_f32(const float* p, float (&v)[N])
{
    if constexpr (N % 4 == 0) {
#pragma unroll
        for (int k = 0; k < N; k += 4) {
            const float4 x = *reinterpret_cast<const float4*>(p + k);
            v[k] = x.x;
            v[k + 1] = x.y;
            v[k + 2] = x.z;
            v[k + 3] = x.w;
        }
    } else if constexpr (N == 2) {
        const float2 x = *reinterpret_cast<const float2*>(p);
        v[0] = x.x;
        v[1] = x.y;
    } else {
        static_assert(N == 1, "accumulator pieces of 1, 2 or a multiple of 4 values");
        v[0] = p[0];
    }
}
template <int N>
__device__ inline void store_f32(float* p, const float (&v)[N])
{
    if constexpr (N % 4 == 0) {
#pragma unroll
        for (int k = 0; k < N; k += 4)
            *reinterpret_cast<float4*>(p + k) = make_float4(v[k], v[k + 1], v[k + 2], v[k + 3]);
    } else if constexpr (N == 2) {
        *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
    } else {
        p[0] = v[0];
    }
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ inline float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Sum over the `width` (power of two, <= 64) consecutive lanes that hold one
// head; every lane of the group receives the total.
__device__ inline float group_sum_pow2(float v, int width)
{
    for (int o = 1; o < width; o <<= 1) v += __shfl_xor(v, o);
    return v;
}

// Sum over `width` consecutive lanes starting at lane `first` for any width.
__device__ inline float group_sum_any(float v, int first, int width)
{
    float s = 0.f;
    for (int k = 0; k < width; ++k) s += __shfl(v, first + k);
    return s;
}

__device__ inline bool is_pow2(int x) { return (x & (x - 1)) == 0; }

// Geometry of one lane inside the row mapping.
template <typename T, int G>
struct LaneMap {
    static constexpr int VEC = Vec<T>::N;
    static constexpr int SLOTS = kWave / G;
    int lane, gl, slot;   // lane in wave, lane in group, group index
    int h;                // head owned by this lane (clamped for idle lanes)
    int lph;              // lanes per head = D / VEC
    int head_first;       // first lane (in wave) of this lane's head group
    bool on;              // lane covers real features
    __device__ inline LaneMap(int F, int H, int D)
    {
        lane = threadIdx.x & (kWave - 1);
        gl = lane & (G - 1);
        slot = lane / G;
        on = gl * VEC < F;
        lph = D / VEC;
        const int hh = (gl * VEC) / D;
        h = hh < H ? hh : H - 1;
        head_first = slot * G + h * lph;
    }
};

// Largest lane piece (in values) that divides a head (or row) width w: 4, 2, 1 for fp32 rows,
// 8, 4, 2, 1 for bf16 rows.
inline int piece_for(int dtype_is_f32, int w)
{
    for (int v = dtype_is_f32 ? 4 : 8; v > 1; v >>= 1)
        if (w % v == 0) return v;
    return 1;
}

// Runs `...` with T bound to the row type of (dtype, piece).
#define SAR_DISPATCH_ROW(dtype, piece, ...)                  \
    do {                                                     \
        if ((dtype) == SAR_F32) {                            \
            if ((piece) == 4) {                              \
                using T = float;                             \
                __VA_ARGS__;                                 \
            } else if ((piece) == 2) {                       \
                using T = ::sar::f32x2_t;                    \
                __VA_ARGS__;                                 \
            } else {                                         \
                using T = ::sar::f32x1_t;                    \
                __VA_ARGS__;                                 \
            }                                                \
        } else {                                             \
            if ((piece) == 8) {                              \
                using T = ::sar::bf16_t;                     \
                __VA_ARGS__;                                 \
            } else if ((piece) == 4) {                       \
                using T = ::sar::bf16x4_t;                   \
                __VA_ARGS__;                                 \
            } else if ((piece) == 2) {                       \
                using T = ::sar::bf16x2_t;                   \
                __VA_ARGS__;                                 \
            } else {                                         \
                using T = ::sar::bf16x1_t;                   \
                __VA_ARGS__;                                 \
            }                                                \
        }                                                    \
    } while (0)

template <typename T>
struct is_full_row {
    static constexpr bool value = false;
};
template <>
struct is_full_row<float> {
    static constexpr bool value = true;
};
template <>
struct is_full_row<bf16_t> {
    static constexpr bool value = true;
};

inline int lanes_for(int F, int vec)
{
    int need = (F + vec - 1) / vec, g = 4;
    while (g < need) g <<= 1;
    return g;
}

}  // namespace sar
