// The dense node-wise transform of Eq. 1 (z = W h, row-major Z = X W) and its
// backward (what Z.backward(E) does in Alg. 2: dW = X^T dZ, dX = dZ W^T) on the
// gfx950 matrix cores.  This is the one real contraction on the path.
//
// One tiled GEMM kernel C = A B serves the three products through strides.
// Operands are widened to fp32 while being staged in LDS and multiplied with
// V_MFMA_F32_32X32X2_F32 (fp32 in, fp32 accumulate), so fp32 configurations
// keep fp32 accuracy and bf16-stored operands are multiplied exactly.
// Workgroup tile 128 x 128 x 16, four wavefronts in a 2 x 2 grid, each owning
// a 64 x 64 patch as 2 x 2 MFMA tiles (64 accumulator registers per lane).
#include <algorithm>

#include "gather_common.h"
#include "sar_internal.h"

namespace {

using namespace sar;

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int kPad = 4;
constexpr int kGemmThreads = 256;

typedef float float16_t __attribute__((ext_vector_type(16)));

template <typename T>
__device__ inline float to_f32(T v);
template <>
__device__ inline float to_f32<float>(float v) { return v; }
template <>
__device__ inline float to_f32<bf16_t>(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }

template <typename T>
__device__ inline T from_f32(float v);
template <>
__device__ inline float from_f32<float>(float v) { return v; }
template <>
__device__ inline bf16_t from_f32<bf16_t>(float v) { return bf16_t{(uint16_t)f32_to_bf16_rne(v)}; }

struct GemmArgs {
    const void* A;
    const void* B;
    void* C;
    int64_t M;        // rows of C
    int N;            // cols of C
    int64_t Kd;       // contraction length
    int64_t sa_i, sa_k;   // A(i,k) = A[i*sa_i + k*sa_k]
    int64_t sb_k, sb_j;   // B(k,j) = B[k*sb_k + j*sb_j]
    int64_t ldc;
    int64_t k_slab;   // contraction range per blockIdx.z (split-K); C advances by c_split per slab
    int64_t c_split;
};

// A_K_FAST: consecutive threads walk k when loading A (A is contiguous in k).
// B_K_FAST: same for B.
template <typename TA, typename TB, typename TC, bool A_K_FAST, bool B_K_FAST>
__global__ __launch_bounds__(kGemmThreads) void k_gemm(GemmArgs g)
{
    __shared__ float As[BK][BM + kPad];
    __shared__ float Bs[BK][BN + kPad];
    const TA* A = static_cast<const TA*>(g.A);
    const TB* B = static_cast<const TB*>(g.B);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int64_t k_beg = (int64_t)blockIdx.z * g.k_slab;
    const int64_t k_end = std::min<int64_t>(g.Kd, k_beg + g.k_slab);

    float16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    for (int64_t k0 = k_beg; k0 < k_end; k0 += BK) {
        // stage A[BM x BK] and B[BK x BN], 8 values per thread each
#pragma unroll
        for (int t = 0; t < (BM * BK) / kGemmThreads; ++t) {
            const int e = t * kGemmThreads + tid;
            int i, kk;
            if (A_K_FAST) {
                kk = e % BK;
                i = e / BK;
            } else {
                i = e % BM;
                kk = e / BM;
            }
            float v = 0.f;
            if (m0 + i < g.M && k0 + kk < k_end) v = to_f32<TA>(A[(m0 + i) * g.sa_i + (k0 + kk) * g.sa_k]);
            As[kk][i] = v;
        }
#pragma unroll
        for (int t = 0; t < (BN * BK) / kGemmThreads; ++t) {
            const int e = t * kGemmThreads + tid;
            int j, kk;
            if (B_K_FAST) {
                kk = e % BK;
                j = e / BK;
            } else {
                j = e % BN;
                kk = e / BN;
            }
            float v = 0.f;
            if (n0 + j < g.N && k0 + kk < k_end) v = to_f32<TB>(B[(k0 + kk) * g.sb_k + (int64_t)(n0 + j) * g.sb_j]);
            Bs[kk][j] = v;
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < BK; ks += 2) {
            const int kk = ks + (lane >> 5);
            float a[2], b[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                a[x] = As[kk][wm * 64 + x * 32 + (lane & 31)];
                b[x] = Bs[kk][wn * 64 + x * 32 + (lane & 31)];
            }
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y)
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[x], b[y], acc[x][y], 0, 0, 0);
        }
        __syncthreads();
    }

    // lane holds column (lane % 32); register r holds row 8*(r/4) + 4*(lane/32) + r%4
    TC* C = static_cast<TC*>(g.C) + (int64_t)blockIdx.z * g.c_split;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) {
            const int j = n0 + wn * 64 + y * 32 + (lane & 31);
            if (j >= g.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t i = m0 + wm * 64 + x * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                if (i < g.M) C[i * g.ldc + j] = from_f32<TC>(acc[x][y][r]);
            }
        }
}

// dW[k] += sum over slabs of partial[slab][k]
__global__ __launch_bounds__(256) void k_sum_slabs(const float* __restrict__ partial, int n_slabs, int64_t count,
                                                   float* __restrict__ dW)
{
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < count; k += (int64_t)gridDim.x * 256) {
        float s = 0.f;
        for (int z = 0; z < n_slabs; ++z) s += partial[(int64_t)z * count + k];
        dW[k] += s;
    }
}

constexpr int kMaxSlabs = 256;

int slabs_for(int64_t n, int K, int F)
{
    const int64_t tiles = (int64_t)((K + BM - 1) / BM) * ((F + BN - 1) / BN);
    int64_t want = std::max<int64_t>(1, (1024 + tiles - 1) / tiles);
    want = std::min<int64_t>(want, kMaxSlabs);
    const int64_t by_rows = std::max<int64_t>(1, n / (4 * BK));
    return (int)std::min(want, by_rows);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" int sar_linear_workspace_bytes(int64_t n, int K, int F, size_t* bytes)
{
    SAR_CHECK_ARG(bytes != nullptr, "bytes is null");
    SAR_CHECK_ARG(n >= 0 && K > 0 && F > 0, "need n >= 0, K > 0, F > 0");
    *bytes = (size_t)slabs_for(n, K, F) * K * F * sizeof(float);
    return SAR_OK;
}

extern "C" int sar_linear_fwd(const void* X, const float* W, void* Z, int dtype, int64_t n, int K, int F, int H,
                              int D, const float* a_score, float* score, const float* a_score2, float* score2,
                              void* stream)
{
    if (dtype != SAR_F32 && dtype != SAR_BF16)
        return sar::fail(SAR_ERR_UNSUPPORTED, "dtype %d is neither SAR_F32 nor SAR_BF16", dtype);
    SAR_CHECK_ARG(n >= 0 && K > 0 && F > 0, "need n >= 0, K > 0, F > 0");
    SAR_CHECK_ARG((a_score == nullptr) == (score == nullptr), "a_score and score must be given together");
    SAR_CHECK_ARG((a_score2 == nullptr) == (score2 == nullptr), "a_score2 and score2 must be given together");
    SAR_CHECK_ARG(!(a_score || a_score2) || (H > 0 && D > 0 && H * D == F), "scores need H*D == F");
    if (n == 0) return SAR_OK;
    SAR_CHECK_ARG(X && W && Z, "X, W or Z is null");
    hipStream_t st = sar::as_stream(stream);
    GemmArgs g{};
    g.A = X;
    g.B = W;
    g.C = Z;
    g.M = n;
    g.N = F;
    g.Kd = K;
    g.sa_i = K;
    g.sa_k = 1;
    g.sb_k = F;
    g.sb_j = 1;
    g.ldc = F;
    g.k_slab = K;
    g.c_split = 0;
    dim3 grid((unsigned)((n + BM - 1) / BM), (unsigned)((F + BN - 1) / BN), 1);
    if (dtype == SAR_F32)
        k_gemm<float, float, float, true, false><<<grid, kGemmThreads, 0, st>>>(g);
    else
        k_gemm<bf16_t, float, bf16_t, true, false><<<grid, kGemmThreads, 0, st>>>(g);
    SAR_LAUNCH_CHECK();
    if (a_score) SAR_TRY(sar_gat_scores(Z, dtype, n, H, D, a_score, score, stream));
    if (a_score2) SAR_TRY(sar_gat_scores(Z, dtype, n, H, D, a_score2, score2, stream));
    return SAR_OK;
}

extern "C" int sar_linear_bwd(const void* X, const void* dZ, const float* W, float* dW, void* dX, int dtype,
                              int64_t n, int K, int F, void* work, size_t work_bytes, void* stream)
{
    if (dtype != SAR_F32 && dtype != SAR_BF16)
        return sar::fail(SAR_ERR_UNSUPPORTED, "dtype %d is neither SAR_F32 nor SAR_BF16", dtype);
    SAR_CHECK_ARG(n >= 0 && K > 0 && F > 0, "need n >= 0, K > 0, F > 0");
    if (n == 0) return SAR_OK;
    SAR_CHECK_ARG(dZ != nullptr, "dZ is null");
    SAR_CHECK_ARG(dW == nullptr || X != nullptr, "dW needs X");
    SAR_CHECK_ARG(dX == nullptr || W != nullptr, "dX needs W");
    hipStream_t st = sar::as_stream(stream);
    if (dW) {
        const int slabs = slabs_for(n, K, F);
        const size_t need = (size_t)slabs * K * F * sizeof(float);
        SAR_CHECK_ARG(work != nullptr && work_bytes >= need, "work_bytes=%zu is below the %zu bytes required",
                      work_bytes, need);
        // dW[K,F] = X^T dZ, contraction over the n rows, split into slabs
        GemmArgs g{};
        g.A = X;
        g.B = dZ;
        g.C = work;
        g.M = K;
        g.N = F;
        g.Kd = n;
        g.sa_i = 1;
        g.sa_k = K;
        g.sb_k = F;
        g.sb_j = 1;
        g.ldc = F;
        g.k_slab = ((n + slabs - 1) / slabs + BK - 1) / BK * BK;
        g.c_split = (int64_t)K * F;
        dim3 grid((unsigned)((K + BM - 1) / BM), (unsigned)((F + BN - 1) / BN), (unsigned)slabs);
        if (dtype == SAR_F32)
            k_gemm<float, float, float, false, false><<<grid, kGemmThreads, 0, st>>>(g);
        else
            k_gemm<bf16_t, bf16_t, float, false, false><<<grid, kGemmThreads, 0, st>>>(g);
        SAR_LAUNCH_CHECK();
        const int64_t count = (int64_t)K * F;
        k_sum_slabs<<<(unsigned)std::min<int64_t>((count + 255) / 256, 4096), 256, 0, st>>>(
            static_cast<const float*>(work), slabs, count, dW);
        SAR_LAUNCH_CHECK();
    }
    if (dX) {
        // dX[n,K] = dZ W^T : B(k=f, j=kcol) = W[kcol*F + f]
        GemmArgs g{};
        g.A = dZ;
        g.B = W;
        g.C = dX;
        g.M = n;
        g.N = K;
        g.Kd = F;
        g.sa_i = F;
        g.sa_k = 1;
        g.sb_k = 1;
        g.sb_j = F;
        g.ldc = K;
        g.k_slab = F;
        g.c_split = 0;
        dim3 grid((unsigned)((n + BM - 1) / BM), (unsigned)((K + BN - 1) / BN), 1);
        if (dtype == SAR_F32)
            k_gemm<float, float, float, true, true><<<grid, kGemmThreads, 0, st>>>(g);
        else
            k_gemm<bf16_t, float, bf16_t, true, true><<<grid, kGemmThreads, 0, st>>>(g);
        SAR_LAUNCH_CHECK();
    }
    return SAR_OK;
}
