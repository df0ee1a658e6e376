// The dense node-wise transform of Eq. 1 (z = W h, row-major Z = X W) and its
// backward (what Z.backward(E) does in Alg. 2: dW = X^T dZ, dX = dZ W^T) on the
// gfx950 matrix cores.  This is the one real contraction on the path.
//
// One tiled GEMM kernel C = A B serves the three products through strides.
// Operands are widened to fp32 while being staged in LDS and multiplied with
// V_MFMA_F32_32X32X2_F32 (fp32 in, fp32 accumulate), so fp32 configurations
// keep fp32 accuracy; bf16-stored operands go through V_MFMA_F32_32X32X16_BF16
// (see below).  Z = X W and dX = dZ W^T normally take the skinny kernel further
// down (small operand resident in LDS, big operand straight into registers);
// the tiled kernel remains for dW and for shapes the skinny one does not cover.
// Workgroup tile 128 x 128 x 32, four wavefronts in a 2 x 2 grid,
// each owning a 64 x 64 patch as 2 x 2 MFMA tiles (64 accumulator registers per
// lane); the next tile is fetched into registers while the current one is
// multiplied.
#include <algorithm>

#include "gather_common.h"
#include "sar_internal.h"

namespace {

using namespace sar;

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int kPad = 4;
constexpr int kGemmThreads = 256;
constexpr int kPerThread = BM * BK / kGemmThreads / 4;   // 4-element groups each thread stages per operand

typedef float float16_t __attribute__((ext_vector_type(16)));

__device__ inline float bf16_to_f32(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }

template <typename T>
__device__ inline T from_f32(float v);
template <>
__device__ inline float from_f32<float>(float v) { return v; }
template <>
__device__ inline bf16_t from_f32<bf16_t>(float v) { return bf16_t{(uint16_t)f32_to_bf16_rne(v)}; }

// four consecutive elements, widened to fp32 (vector access when `vec`)
template <typename T>
__device__ inline void load4(const T* p, bool vec, int n_valid, float (&v)[4]);
template <>
__device__ inline void load4<float>(const float* p, bool vec, int n_valid, float (&v)[4])
{
    if (vec && n_valid == 4) {
        const float4 x = *reinterpret_cast<const float4*>(p);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = k < n_valid ? p[k] : 0.f;
    }
}
template <>
__device__ inline void load4<bf16_t>(const bf16_t* p, bool vec, int n_valid, float (&v)[4])
{
    if (vec && n_valid == 4) {
        const uint2 x = *reinterpret_cast<const uint2*>(p);
        v[0] = __uint_as_float(x.x << 16);
        v[1] = __uint_as_float(x.x & 0xffff0000u);
        v[2] = __uint_as_float(x.y << 16);
        v[3] = __uint_as_float(x.y & 0xffff0000u);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = k < n_valid ? bf16_to_f32(p[k]) : 0.f;
    }
}

struct GemmArgs {
    const void* A;
    const void* B;
    void* C;
    int64_t M;        // rows of C
    int N;            // cols of C
    int64_t Kd;       // contraction length
    int64_t lda;      // A_K_FAST: A(i,k) = A[i*lda + k]   else A(i,k) = A[k*lda + i]
    int64_t ldb;      // B_K_FAST: B(k,j) = B[j*ldb + k]   else B(k,j) = B[k*ldb + j]
    int64_t ldc;
    int64_t k_slab;   // contraction range per blockIdx.z (split-K); C advances by c_split per slab
    int64_t c_split;
    int vec_a, vec_b; // 4-element groups of A / B are aligned and in one row
};

// One operand tile of TILE x BK (TILE = BM or BN) staged through registers:
// each thread owns kPerThread groups of 4 elements that are consecutive in the
// operand's contiguous dimension (k when K_FAST, else the tile dimension).
template <typename T, bool K_FAST>
struct Stage {
    float v[kPerThread][4];
    __device__ inline void fetch(const T* base, int64_t ld, int64_t x0, int64_t x_end, int64_t k0, int64_t k_end,
                                 bool vec, int tid)
    {
#pragma unroll
        for (int g = 0; g < kPerThread; ++g) {
            const int e = g * kGemmThreads + tid;
            if (K_FAST) {
                const int kk = (e % (BK / 4)) * 4, x = e / (BK / 4);
                const int64_t nk = k_end - (k0 + kk);
                const int nv = (x0 + x < x_end) ? (int)(nk >= 4 ? 4 : (nk > 0 ? nk : 0)) : 0;
                if (nv > 0)
                    load4<T>(base + (x0 + x) * ld + k0 + kk, vec, nv, v[g]);
                else
                    v[g][0] = v[g][1] = v[g][2] = v[g][3] = 0.f;
            } else {
                const int x = (e % (BM / 4)) * 4, kk = e / (BM / 4);
                const int64_t nx = x_end - (x0 + x);
                const int nv = (k0 + kk < k_end) ? (int)(nx >= 4 ? 4 : (nx > 0 ? nx : 0)) : 0;
                if (nv > 0)
                    load4<T>(base + (k0 + kk) * ld + x0 + x, vec, nv, v[g]);
                else
                    v[g][0] = v[g][1] = v[g][2] = v[g][3] = 0.f;
            }
        }
    }
    __device__ inline void commit(float (*tile)[BM + kPad], int tid) const
    {
#pragma unroll
        for (int g = 0; g < kPerThread; ++g) {
            const int e = g * kGemmThreads + tid;
            if (K_FAST) {
                const int kk = (e % (BK / 4)) * 4, x = e / (BK / 4);
#pragma unroll
                for (int c = 0; c < 4; ++c) tile[kk + c][x] = v[g][c];
            } else {
                const int x = (e % (BM / 4)) * 4, kk = e / (BM / 4);
                *reinterpret_cast<float4*>(&tile[kk][x]) = make_float4(v[g][0], v[g][1], v[g][2], v[g][3]);
            }
        }
    }
};

static_assert(BM == BN, "operand staging assumes square workgroup tiles");

// A_K_FAST: A is contiguous along the contraction; B_K_FAST: same for B.
template <typename TA, typename TB, typename TC, bool A_K_FAST, bool B_K_FAST>
__global__ __launch_bounds__(kGemmThreads) void k_gemm(GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) float As[BK][BM + kPad];
    __shared__ __attribute__((aligned(16))) float Bs[BK][BN + kPad];
    const TA* A = static_cast<const TA*>(g.A);
    const TB* B = static_cast<const TB*>(g.B);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int64_t n0 = (int64_t)blockIdx.y * BN;
    const int64_t k_beg = (int64_t)blockIdx.z * g.k_slab;
    const int64_t k_end = std::min<int64_t>(g.Kd, k_beg + g.k_slab);

    float16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    Stage<TA, A_K_FAST> sa;
    Stage<TB, B_K_FAST> sb;
    if (k_beg < k_end) {
        sa.fetch(A, g.lda, m0, g.M, k_beg, k_end, g.vec_a, tid);
        sb.fetch(B, g.ldb, n0, g.N, k_beg, k_end, g.vec_b, tid);
    }
    for (int64_t k0 = k_beg; k0 < k_end; k0 += BK) {
        sa.commit(As, tid);
        sb.commit(Bs, tid);
        __syncthreads();
        // the next tile travels from HBM while this one is multiplied
        if (k0 + BK < k_end) {
            sa.fetch(A, g.lda, m0, g.M, k0 + BK, k_end, g.vec_a, tid);
            sb.fetch(B, g.ldb, n0, g.N, k0 + BK, k_end, g.vec_b, tid);
        }
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
            const int64_t j = n0 + wn * 64 + y * 32 + (lane & 31);
            if (j >= g.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t i = m0 + wm * 64 + x * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                if (i < g.M) C[i * g.ldc + j] = from_f32<TC>(acc[x][y][r]);
            }
        }
}

// ---- bf16-stored operands: bf16 MFMA --------------------------------------
//
// With bf16 storage the products are exact in a bf16 MFMA with fp32
// accumulation, at several times the fp32 MFMA rate.  The fp32 weight matrix is
// split into two bf16 terms, W = hi + lo (+ an error below 2^-17 |W|), and
// multiplied in two instructions, which is far below the bf16 rounding of the
// stored result.  Tiles are staged in LDS as bf16 with the contraction index
// contiguous, the layout V_MFMA_F32_32X32X16_BF16 wants: lane l supplies
// A[l%32][8*(l/32) .. +7] and B[8*(l/32) .. +7][l%32].

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
constexpr int kPadH = 8;

template <bool K_FAST>
__device__ inline void commit_bf16(const float (&v)[kPerThread][4], uint16_t (*hi)[BK + kPadH],
                                   uint16_t (*lo)[BK + kPadH], int tid)
{
#pragma unroll
    for (int g = 0; g < kPerThread; ++g) {
        const int e = g * kGemmThreads + tid;
        uint32_t h[4], l[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            h[c] = f32_to_bf16_rne(v[g][c]);
            l[c] = lo ? f32_to_bf16_rne(v[g][c] - __uint_as_float(h[c] << 16)) : 0u;
        }
        if (K_FAST) {
            const int kk = (e % (BK / 4)) * 4, x = e / (BK / 4);
            *reinterpret_cast<uint2*>(&hi[x][kk]) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
            if (lo) *reinterpret_cast<uint2*>(&lo[x][kk]) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
        } else {
            const int x = (e % (BM / 4)) * 4, kk = e / (BM / 4);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                hi[x + c][kk] = (uint16_t)h[c];
                if (lo) lo[x + c][kk] = (uint16_t)l[c];
            }
        }
    }
}

template <typename TA, typename TB, typename TC, bool A_K_FAST, bool B_K_FAST, bool SPLIT_B>
__global__ __launch_bounds__(kGemmThreads) void k_gemm_bf16(GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) uint16_t As[BM][BK + kPadH];
    __shared__ __attribute__((aligned(16))) uint16_t Bh[BN][BK + kPadH];
    __shared__ __attribute__((aligned(16))) uint16_t Bl[SPLIT_B ? BN : 1][BK + kPadH];
    const TA* A = static_cast<const TA*>(g.A);
    const TB* B = static_cast<const TB*>(g.B);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int64_t n0 = (int64_t)blockIdx.y * BN;
    const int64_t k_beg = (int64_t)blockIdx.z * g.k_slab;
    const int64_t k_end = std::min<int64_t>(g.Kd, k_beg + g.k_slab);

    float16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    Stage<TA, A_K_FAST> sa;
    Stage<TB, B_K_FAST> sb;
    if (k_beg < k_end) {
        sa.fetch(A, g.lda, m0, g.M, k_beg, k_end, g.vec_a, tid);
        sb.fetch(B, g.ldb, n0, g.N, k_beg, k_end, g.vec_b, tid);
    }
    for (int64_t k0 = k_beg; k0 < k_end; k0 += BK) {
        commit_bf16<A_K_FAST>(sa.v, As, nullptr, tid);
        commit_bf16<B_K_FAST>(sb.v, Bh, SPLIT_B ? Bl : nullptr, tid);
        __syncthreads();
        if (k0 + BK < k_end) {
            sa.fetch(A, g.lda, m0, g.M, k0 + BK, k_end, g.vec_a, tid);
            sb.fetch(B, g.ldb, n0, g.N, k0 + BK, k_end, g.vec_b, tid);
        }
#pragma unroll
        for (int ks = 0; ks < BK; ks += 16) {
            const int kk = ks + 8 * (lane >> 5);
            bf16x8_t a[2], bh[2], bl[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                a[x] = *reinterpret_cast<const bf16x8_t*>(&As[wm * 64 + x * 32 + (lane & 31)][kk]);
                bh[x] = *reinterpret_cast<const bf16x8_t*>(&Bh[wn * 64 + x * 32 + (lane & 31)][kk]);
                if (SPLIT_B) bl[x] = *reinterpret_cast<const bf16x8_t*>(&Bl[wn * 64 + x * 32 + (lane & 31)][kk]);
            }
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y) {
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x], bh[y], acc[x][y], 0, 0, 0);
                    if (SPLIT_B) acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x], bl[y], acc[x][y], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    TC* C = static_cast<TC*>(g.C) + (int64_t)blockIdx.z * g.c_split;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) {
            const int64_t j = n0 + wn * 64 + y * 32 + (lane & 31);
            if (j >= g.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t i = m0 + wm * 64 + x * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                if (i < g.M) C[i * g.ldc + j] = from_f32<TC>(acc[x][y][r]);
            }
        }
}

// ---- error rows that are never stored ---------------------------------------
//
// Z_p.backward(E_p) of Alg. 2 reads the worker's error E_p twice (dW = X^T E_p, dX = E_p W^T).
// For the attention layer E_p = E_{p->p} + ds (x) a_r: the local block's error, stored compactly
// (one row per touched source), plus a rank-one term per head.  Instead of writing that sum out
// and reading it back twice, the two products can form each 16-byte piece of it where they load
// the operand: piece(i, f..) = E[row of i][f..] (zero where E has no row for i) + ds[i, f/D] a_r[f..],
// in fp32 and rounded to the storage type exactly as a stored E_p would have been.
struct RowsOp {
    const int32_t* rank;   // [n+1]: node i's row of E is rank[i], present iff rank[i+1] > rank[i]; null: row i
    const float* ds;       // [n, H] or null (no rank-one term)
    const float* a_r;      // [H*D]
    int H, D;
    int has_E;             // 0: E has no rows at all (or is null)
};

template <typename T>
__device__ inline uint4 fuse_piece(const uint4& base, float d, const float* ar);
template <>
__device__ inline uint4 fuse_piece<float>(const uint4& base, float d, const float* ar)
{
    return make_uint4(__float_as_uint(fmaf(d, ar[0], __uint_as_float(base.x))),
                      __float_as_uint(fmaf(d, ar[1], __uint_as_float(base.y))),
                      __float_as_uint(fmaf(d, ar[2], __uint_as_float(base.z))),
                      __float_as_uint(fmaf(d, ar[3], __uint_as_float(base.w))));
}
template <>
__device__ inline uint4 fuse_piece<bf16_t>(const uint4& base, float d, const float* ar)
{
    float v[8];
    Vec<bf16_t>::unpack(base, v);
#pragma unroll
    for (int x = 0; x < 8; ++x) v[x] = fmaf(d, ar[x], v[x]);
    uint4 r;
    r.x = pack2_bf16(v[0], v[1]);
    r.y = pack2_bf16(v[2], v[3]);
    r.z = pack2_bf16(v[4], v[5]);
    r.w = pack2_bf16(v[6], v[7]);
    return r;
}

// ---- skinny products: the small operand resident in LDS --------------------
//
// In Z = X W and dX = dZ W^T the left operand has millions of rows whose
// contraction index is contiguous in memory, which is exactly what an MFMA A
// fragment wants from a lane: lane l of a 32-row tile supplies row l%32 and a
// 16-byte piece of it (4 floats or 8 bf16 values) chosen by l/32.  So the big
// operand goes from HBM straight into registers, never through LDS.  The small
// operand (at most a few hundred KB) is laid out in LDS once per workgroup, in
// the order the B fragments are consumed: one 16-byte unit per lane, 64 units
// per fragment, so every ds_read_b128 is conflict-free.  After that one
// barrier the wavefronts never synchronise again: each walks over its own
// 32-row tiles, keeping NT 32x32 accumulators (32 x NT*32 outputs) in
// registers and two pairs of 16-byte pieces of its rows, one in flight while the other is used.
//
// fp32: a chunk is 8 contraction values; lane group g = l/32 holds values
//       8t+4g .. 8t+4g+3, consumed by four V_MFMA_F32_32X32X2_F32 (whose A and
//       B operands both take "their k" from the lane group, so any pairing of
//       k with (step, group) is valid as long as both operands use the same).
// bf16: a chunk is 16 values, one V_MFMA_F32_32X32X16_BF16 per bf16 half of the
//       fp32 small operand (hi and lo, as above).

constexpr int kSkinnyWaves = 8;
constexpr int kSkinnyThreads = 64 * kSkinnyWaves;
constexpr size_t kSkinnyMaxLds = 160 * 1024;   // all of a CU's LDS: one workgroup per CU then

struct SkinnyArgs {
    const void* A;     // [M, K], row stride lda, contraction index contiguous
    int64_t lda, M;
    const float* B;    // B(k, n) = B[k * sbk + n * sbn]
    int64_t sbk, sbn;
    void* C;           // [M, N], row stride ldc
    int64_t ldc;
    int K, N;
    int chunks;        // ceil(K / chunk length)
    // score projections (Eq. 3: the two halves of a^T (z_i || z_j)) as one more
    // accumulator tile: column h of it is x . (W_h a1_h), column H+h is x . (W_h a2_h)
    const float* a1;   // [H, D] or null
    const float* a2;
    float* s1;         // [M, H] or null
    float* s2;
    int H, D;
    // byte offset in LDS of the per-wavefront 32 x 32 staging tiles through which the outputs
    // are stored as whole 64- or 128-byte row segments, or 0 to store element-wise
    int stage_off;
    RowsOp op;         // FUSE only: how the rows of A are formed
};


// FUSE: the rows of A are not stored; each piece is formed where it is multiplied (RowsOp, K <= 256).
// Between the epilogues a wavefront's staging tile is idle, so it holds what the pieces need: the
// tile's 32 x H values of ds and the K values of a_r.  The row map and ds of a tile are read one
// tile ahead (the map two), like the first pieces of its rows.
constexpr int kDsRegs = 8;   // 32 rows x H <= 16 heads of ds, 64 lanes

template <typename TA, typename TC, int NT, bool SC, bool FUSE = false>
__global__ __launch_bounds__(kSkinnyThreads) void k_gemm_skinny(SkinnyArgs g)
{
    static_assert(!(SC && FUSE), "the fused operand is that of dX = E W^T, which has no score columns");
    constexpr int NA = NT + (SC ? 1 : 0);   // accumulator tiles: NT of the product, one of scores
    extern __shared__ __attribute__((aligned(16))) unsigned char skinny_lds[];
    constexpr bool BF = sizeof(TA) == 2;
    constexpr int kChunk = BF ? 16 : 8;
    constexpr int kFragsPerTile = BF ? 2 : 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, gq = lane >> 5;
    const int64_t n0 = (int64_t)blockIdx.y * (NT * 32);
    uint4* frag = reinterpret_cast<uint4*>(skinny_lds);

    const int units = g.chunks * NA * kFragsPerTile * 64;
    auto make_frag = [&](int u) -> uint4 {
        const int l = u & 63;
        int f = u >> 6, half = 0;
        if (BF) {
            half = f & 1;
            f >>= 1;
        }
        const int nt = f % NA, t = f / NA;
        // the score tile starts as zeros; its entries are written below
        const int64_t n = (SC && nt == NT) ? g.N : n0 + nt * 32 + (l & 31);
        const int kb = t * kChunk + (l >> 5) * (kChunk / 2);
        uint32_t w[4];
        if (!BF) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                w[j] = (kb + j < g.K && n < g.N) ? __float_as_uint(g.B[(int64_t)(kb + j) * g.sbk + n * g.sbn]) : 0u;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t part[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int k = kb + 2 * j + e;
                    const float v = (k < g.K && n < g.N) ? g.B[(int64_t)k * g.sbk + n * g.sbn] : 0.f;
                    const uint32_t hi = f32_to_bf16_rne(v);
                    part[e] = half ? f32_to_bf16_rne(v - __uint_as_float(hi << 16)) : hi;
                }
                w[j] = part[0] | (part[1] << 16);
            }
        }
        return make_uint4(w[0], w[1], w[2], w[3]);
    };
    // four fragments per thread and round, so that their 16 loads travel together
    for (int u0 = tid; u0 < units; u0 += 4 * kSkinnyThreads) {
        uint4 val[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) val[x] = make_frag(min(u0 + x * kSkinnyThreads, units - 1));
#pragma unroll
        for (int x = 0; x < 4; ++x)
            if (u0 + x * kSkinnyThreads < units) frag[u0 + x * kSkinnyThreads] = val[x];
    }
    if (SC) {
        // (W a)[k][h] = sum_d W[k][h*D + d] a[h][d]: z_h . a_h = x . (W_h a_h), so the scores
        // are 2H more output columns of the same product, taken from the unrounded sums
        __syncthreads();
        // a head's two score columns belong to the column slab that holds the head's first
        // column; the other slabs leave them at zero and do not store them
        const int cols = 2 * g.H;
        for (int p = tid; p < g.K * cols; p += kSkinnyThreads) {
            const int k = p / cols, col = p % cols;
            const int h = col < g.H ? col : col - g.H;
            const float* av = col < g.H ? g.a1 : g.a2;
            const int t = k / kChunk, gk = (k / (kChunk / 2)) & 1, e = k % (kChunk / 2);
            float v = 0.f;
            if (av && (h * g.D) / (NT * 32) == (int)blockIdx.y) {
                if (!BF && (int64_t)(h + 1) * g.D <= n0 + NT * 32) {
                    // this head's part of row k of W is in LDS already (exact fp32 values, fragment
                    // order): D strided reads of global memory per product would cost more than
                    // the whole staging
                    const float* wk = reinterpret_cast<const float*>(frag) + ((size_t)t * NA * 64 + gk * 32) * 4 + e;
                    for (int d = 0; d < g.D; ++d) {
                        const int n = h * g.D + d - (int)n0;
                        v = fmaf(wk[((n >> 5) * 64 + (n & 31)) * 4], av[h * g.D + d], v);
                    }
                } else {
                    const float* wrow = g.B + (int64_t)k * g.sbk + (int64_t)h * g.D * g.sbn;
                    for (int d = 0; d < g.D; ++d) v = fmaf(wrow[d * g.sbn], av[h * g.D + d], v);
                }
            }
            if (!BF) {
                reinterpret_cast<float*>(frag)[(((size_t)t * NA + NT) * 64 + gk * 32 + col) * 4 + e] = v;
            } else {
                uint16_t* fh = reinterpret_cast<uint16_t*>(frag);
                const uint32_t hi = f32_to_bf16_rne(v);
                const size_t at = ((size_t)t * NA + NT) * 2 * 64 + gk * 32 + col;
                fh[at * 8 + e] = (uint16_t)hi;
                fh[(at + 64) * 8 + e] = (uint16_t)f32_to_bf16_rne(v - __uint_as_float(hi << 16));
            }
        }
    }
    __syncthreads();

    const TA* A = static_cast<const TA*>(g.A);
    const int64_t n_tiles = (g.M + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * kSkinnyWaves;
    int64_t tile = (int64_t)blockIdx.x * kSkinnyWaves + wave;
    if (tile >= n_tiles) return;

    // K is a multiple of the lane's piece, so a piece is inside the row or beyond it.  Loads are
    // unconditional (a piece beyond the row is read from the row's last piece, and zeroed where it
    // is used) and the main loop below is straight-line code, so that the compiler can count the
    // loads in flight and wait for the oldest only; with branches around them it waits for all of
    // them at every chunk, which leaves the ring no depth.
    const int k_last = g.K - kChunk / 2;
    auto load_piece = [&](const TA* rowp, int t) -> uint4 {
        const int k = t * kChunk + gq * (kChunk / 2);
        return *reinterpret_cast<const uint4*>(rowp + min(k, k_last));
    };
    auto row_ptr = [&](int64_t tl) { return A + std::min<int64_t>(tl * 32 + c, g.M - 1) * g.lda; };

    // FUSE: where this lane's row of the stored part is (row 0, and `has` false, where there is none:
    // the loads stay unconditional), the tile's ds values on their way to LDS, the lane's four a_r
    float* dsl = nullptr;
    float* arl = nullptr;
    float arreg[4] = {0.f, 0.f, 0.f, 0.f}, dsreg[kDsRegs];
    int nrk0 = 0, nrk1 = 0;
    bool has = false;
    const float inv_D = FUSE ? 1.f / (float)g.op.D : 0.f;
    auto rank_of = [&](int64_t tl, int& r0, int& r1) {
        if (g.op.rank && tl < n_tiles) {
            const int64_t i = std::min<int64_t>(tl * 32 + c, g.M - 1);
            r0 = g.op.rank[i];
            r1 = g.op.rank[i + 1];
        }
    };
    auto row_ptr_fused = [&](int64_t tl, int r0, int r1, bool& present) -> const TA* {
        if (!g.op.has_E) {
            present = false;
            return A;                      // a readable stand-in row
        }
        if (g.op.rank) {
            present = r1 > r0;
            return A + (int64_t)(present ? r0 : 0) * g.lda;
        }
        present = true;
        return row_ptr(tl);
    };
    auto load_ds = [&](int64_t tl) {
        const int64_t first = tl * 32 * g.op.H, end = g.M * g.op.H;
#pragma unroll
        for (int r = 0; r < kDsRegs; ++r) {
            const int idx = lane + 64 * r;
            dsreg[r] = (g.op.ds && idx < 32 * g.op.H && first + idx < end) ? g.op.ds[first + idx] : 0.f;
        }
    };
    if constexpr (FUSE) {
        dsl = reinterpret_cast<float*>(skinny_lds + g.stage_off + wave * (32 * 32 * (int)sizeof(TC)));
        arl = dsl + 32 * g.op.H;
#pragma unroll
        for (int x = 0; x < 4; ++x) arreg[x] = (g.op.ds && lane * 4 + x < g.K) ? g.op.a_r[lane * 4 + x] : 0.f;
    }

    // Two sets of pieces: while the chunks of one set are multiplied, the other set travels.
    // The loads of a set are issued together, ahead of the other set's MFMAs, and are first
    // needed a whole set later.  (The compiler waits for every load in flight, not for the oldest,
    // wherever stores may be in flight too, so a deeper ring of single loads gains nothing.)
    // chunks per set: about 2000 MFMA cycles of one wavefront either way (two where registers run out)
    constexpr int PS = (BF && !(SC && NT == 8)) ? 4 : 2;
    uint4 a[PS], b[PS];
    const TA* rowp;
    if constexpr (FUSE) {
        rank_of(tile, nrk0, nrk1);
        rowp = row_ptr_fused(tile, nrk0, nrk1, has);
        load_ds(tile);
        rank_of(tile + stride, nrk0, nrk1);
    } else {
        rowp = row_ptr(tile);
    }
#pragma unroll
    for (int u = 0; u < PS; ++u) a[u] = load_piece(rowp, u);
    const int full = g.chunks / (2 * PS) * (2 * PS);

    for (; tile < n_tiles; tile += stride) {
        float16_t acc[NA];
#pragma unroll
        for (int nt = 0; nt < NA; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nt][r] = 0.f;
        if constexpr (FUSE) {
            // the previous tile's outputs have left the staging tile
            // kept head-major, [H][32 rows]: the 32 rows of a head sit in 32 different banks
#pragma unroll
            for (int r = 0; r < kDsRegs; ++r) {
                const int idx = lane + 64 * r;
                if (idx < 32 * g.op.H) dsl[(idx % g.op.H) * 32 + idx / g.op.H] = dsreg[r];
            }
            *reinterpret_cast<float4*>(arl + lane * 4) = make_float4(arreg[0], arreg[1], arreg[2], arreg[3]);
            __builtin_amdgcn_wave_barrier();
        }

        auto multiply = [&](const uint4& piece, int t) {
            const int k_first = t * kChunk + gq * (kChunk / 2);
            const bool beyond = k_first >= g.K;
            uint4 av = make_uint4(beyond ? 0u : piece.x, beyond ? 0u : piece.y, beyond ? 0u : piece.z,
                                  beyond ? 0u : piece.w);
            if constexpr (FUSE) {
                if (!has) av = make_uint4(0u, 0u, 0u, 0u);
                // a_r is zero beyond K, so a piece beyond the row stays zero
                // head of the piece: k_first / D for 0 <= k_first < 512, without an integer division
                const int head = min((int)(((float)k_first + 0.5f) * inv_D), g.op.H - 1);
                const float d = dsl[head * 32 + c];
                float ar[kChunk / 2];
#pragma unroll
                for (int x = 0; x < kChunk / 2; x += 4) {
                    const float4 v = *reinterpret_cast<const float4*>(arl + k_first + x);
                    ar[x] = v.x; ar[x + 1] = v.y; ar[x + 2] = v.z; ar[x + 3] = v.w;
                }
                av = fuse_piece<TA>(av, d, ar);
            }
            const uint4* fr = frag + (size_t)t * (NA * kFragsPerTile * 64) + lane;
            if (!BF) {
                uint4 w[NA];
#pragma unroll
                for (int nt = 0; nt < NA; ++nt) w[nt] = fr[nt * 64];
#pragma unroll
                for (int nt = 0; nt < NA; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av.x), __uint_as_float(w[nt].x),
                                                                   acc[nt], 0, 0, 0);
#pragma unroll
                for (int nt = 0; nt < NA; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av.y), __uint_as_float(w[nt].y),
                                                                   acc[nt], 0, 0, 0);
#pragma unroll
                for (int nt = 0; nt < NA; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av.z), __uint_as_float(w[nt].z),
                                                                   acc[nt], 0, 0, 0);
#pragma unroll
                for (int nt = 0; nt < NA; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av.w), __uint_as_float(w[nt].w),
                                                                   acc[nt], 0, 0, 0);
            } else {
                const bf16x8_t ax = __builtin_bit_cast(bf16x8_t, av);
#pragma unroll
                for (int nt = 0; nt < NA; ++nt) {
                    const bf16x8_t bh = __builtin_bit_cast(bf16x8_t, fr[(2 * nt) * 64]);
                    acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax, bh, acc[nt], 0, 0, 0);
                }
#pragma unroll
                for (int nt = 0; nt < NA; ++nt) {
                    const bf16x8_t bl = __builtin_bit_cast(bf16x8_t, fr[(2 * nt + 1) * 64]);
                    acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax, bl, acc[nt], 0, 0, 0);
                }
            }
        };
        for (int t0 = 0; t0 < full; t0 += 2 * PS) {
#pragma unroll
            for (int u = 0; u < PS; ++u) b[u] = load_piece(rowp, t0 + PS + u);
            __builtin_amdgcn_sched_barrier(0);     // the loads stay ahead of the MFMAs
#pragma unroll
            for (int u = 0; u < PS; ++u) multiply(a[u], t0 + u);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < PS; ++u) a[u] = load_piece(rowp, t0 + 2 * PS + u);   // beyond the end: nobody reads it
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < PS; ++u) multiply(b[u], t0 + PS + u);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the last chunks, fewer than two sets: the first set is loaded already
        if (full + PS < g.chunks) {
#pragma unroll
            for (int u = 0; u < PS; ++u) b[u] = load_piece(rowp, full + PS + u);
        }
#pragma unroll
        for (int u = 0; u < PS; ++u)
            if (full + u < g.chunks) multiply(a[u], full + u);
#pragma unroll
        for (int u = 0; u < PS; ++u)
            if (full + PS + u < g.chunks) multiply(b[u], full + PS + u);

        // the next tile's first pieces travel while this one is stored
        const int64_t row0 = tile * 32;
        if (tile + stride < n_tiles) {
            if constexpr (FUSE) {
                rowp = row_ptr_fused(tile + stride, nrk0, nrk1, has);
                load_ds(tile + stride);
                rank_of(tile + 2 * stride, nrk0, nrk1);
            } else {
                rowp = row_ptr(tile + stride);
            }
#pragma unroll
            for (int u = 0; u < PS; ++u) a[u] = load_piece(rowp, u);
        }
        // lane holds column c; register r holds row 8*(r/4) + 4*(lane/32) + r%4
        TC* C = static_cast<TC*>(g.C);
        if (g.stage_off) {
            // A lane's 16 values of a tile are 16 different rows: stored directly they are 2- or
            // 4-byte writes, 128 store instructions per 32 x 256 outputs and more of them than a
            // wavefront may have in flight.  The tile is turned through the wavefront's own
            // 2 or 4 KB of LDS instead and leaves as 16-byte pieces, whole 64- or 128-byte rows.
            constexpr int kPer = 16 / (int)sizeof(TC);        // values per piece
            constexpr int kPieces = 32 / kPer;                // pieces per tile row
            constexpr int kRows = 64 / kPieces;               // tile rows per store instruction
            TC* stg = reinterpret_cast<TC*>(skinny_lds + g.stage_off + wave * (32 * 32 * (int)sizeof(TC)));
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    stg[(8 * (r / 4) + 4 * gq + (r % 4)) * 32 + c] = from_f32<TC>(acc[nt][r]);
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int pass = 0; pass < 32 / kRows; ++pass) {
                    const int row = pass * kRows + lane / kPieces, piece = lane % kPieces;
                    const TC* from = stg + row * 32 + piece * kPer;
                    const int64_t i = row0 + row, n = n0 + nt * 32 + piece * kPer;
                    if (i < g.M) {
                        if (n + kPer <= g.N) {
                            *reinterpret_cast<uint4*>(C + i * g.ldc + n) = *reinterpret_cast<const uint4*>(from);
                        } else {
                            for (int e = 0; e < kPer && n + e < g.N; ++e) C[i * g.ldc + n + e] = from[e];
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
        } else {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int64_t n = n0 + nt * 32 + c;
                if (n >= g.N) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t i = row0 + 8 * (r / 4) + 4 * gq + (r % 4);
                    if (i < g.M) C[i * g.ldc + n] = from_f32<TC>(acc[nt][r]);
                }
            }
        }
        if (SC && c < 2 * g.H) {
            float* dst = c < g.H ? g.s1 : g.s2;
            const int h = c < g.H ? c : c - g.H;
            if (dst && (h * g.D) / (NT * 32) == (int)blockIdx.y) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t i = row0 + 8 * (r / 4) + 4 * gq + (r % 4);
                    if (i < g.M) dst[i * g.H + h] = acc[NA - 1][r];
                }
            }
        }
    }
}

struct SkinnyPlan {
    int nt = 0;          // accumulator tiles per workgroup slab (1, 2, 4 or 8)
    unsigned slabs = 0;  // column slabs of nt*32
    size_t lds = 0;
    int chunks = 0;
    int stage_off = 0;   // see SkinnyArgs
};

// Whether the skinny kernel applies: 16-byte pieces of A rows must be aligned
// and whole, and the small operand must fit in LDS in at most four column slabs.
bool plan_skinny(const void* A, int64_t lda, const void* C, int64_t ldc, int K, int N, int dtype, int extra_tiles,
                 SkinnyPlan* p)
{
    const int elem = dtype == SAR_F32 ? 4 : 2, piece = 16 / elem;
    if (reinterpret_cast<uintptr_t>(A) % 16 != 0 || (lda * elem) % 16 != 0 || K % piece != 0) return false;
    const int chunk = 2 * piece;
    p->chunks = (K + chunk - 1) / chunk;
    const size_t unit = dtype == SAR_F32 ? 1024 : 2048;
    const int need = (N + 31) / 32;
    int nt = 1;
    while (nt < need && nt < 8) nt *= 2;
    // Outputs go through staging tiles when their 16-byte pieces are aligned: always for 2-byte
    // outputs (stored directly they are scattered 2-byte writes), for 4-byte outputs when the
    // tiles fit beside the small operand without narrowing the slab
    bool stage = reinterpret_cast<uintptr_t>(C) % 16 == 0 && (ldc * elem) % 16 == 0;
    size_t stage_bytes = stage ? (size_t)kSkinnyWaves * 32 * 32 * elem : 0;
    auto fits = [&](int t, size_t extra) {
        return (size_t)p->chunks * (t + extra_tiles) * unit + extra <= kSkinnyMaxLds;
    };
    if (dtype == SAR_F32) {
        while (nt >= 1 && !fits(nt, 0)) nt /= 2;
        if (nt >= 1 && !fits(nt, stage_bytes)) {
            stage = false;
            stage_bytes = 0;
        }
    } else {
        while (nt >= 1 && !fits(nt, stage_bytes)) nt /= 2;
    }
    if (nt < 1) return false;
    p->nt = nt;
    p->slabs = (unsigned)((need + nt - 1) / nt);
    p->lds = (size_t)p->chunks * (nt + extra_tiles) * unit;
    p->stage_off = stage ? (int)p->lds : 0;
    p->lds += stage_bytes;
    return p->slabs <= 4;
}

template <typename TA, typename TC, int NT, bool SC, bool FUSE = false>
int launch_skinny_nt(const SkinnyArgs& g, const SkinnyPlan& p, hipStream_t st)
{
    int dev = 0;
    SAR_HIP(hipGetDevice(&dev));
    int n_cu = 0;
    SAR_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    SAR_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_skinny<TA, TC, NT, SC, FUSE>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds));
    const int64_t tiles = (g.M + 31) / 32;
    const int64_t want = (tiles + kSkinnyWaves - 1) / kSkinnyWaves;
    // one workgroup per CU; two where registers (NT <= 4) and LDS leave room
    const int per_cu = (NT <= 4 && 2 * p.lds <= 150 * 1024) ? 2 : 1;
    const int64_t resident = std::max<int64_t>(1, (int64_t)n_cu * per_cu / p.slabs);
    dim3 grid((unsigned)std::max<int64_t>(1, std::min(want, resident)), p.slabs, 1);
    k_gemm_skinny<TA, TC, NT, SC, FUSE><<<grid, kSkinnyThreads, p.lds, st>>>(g);
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

template <typename TA, typename TC, bool SC, bool FUSE = false>
int launch_skinny(const SkinnyArgs& g, const SkinnyPlan& p, hipStream_t st)
{
    switch (p.nt) {
        case 1: return launch_skinny_nt<TA, TC, 1, SC, FUSE>(g, p, st);
        case 2: return launch_skinny_nt<TA, TC, 2, SC, FUSE>(g, p, st);
        case 4: return launch_skinny_nt<TA, TC, 4, SC, FUSE>(g, p, st);
        default: return launch_skinny_nt<TA, TC, 8, SC, FUSE>(g, p, st);
    }
}

// Whether a plan can also form the rows of A on the fly (k_gemm_skinny's FUSE): the outputs must
// go through staging tiles, and a tile must hold 32 x H values of ds and 256 of a_r.
bool plan_takes_rows_op(const SkinnyPlan& p, int K, int H, int dtype)
{
    const size_t tile = 32 * 32 * (dtype == SAR_F32 ? 4 : 2);
    // (with eight accumulator tiles the registers are spoken for)
    return p.nt <= 4 && p.stage_off != 0 && K <= 256 && H <= 2 * kDsRegs && (size_t)(32 * H + 256) * 4 <= tile;
}

// ---- dW = X^T dZ: contraction over the rows ---------------------------------
//
// Here both operands have the contraction index (the node) as their slow
// dimension, the opposite of what an MFMA fragment wants from a lane.  A
// workgroup copies chunks of rows of X (up to 128 columns) and dZ (up to 256
// columns) into LDS as they are (16-byte accesses both sides, double
// buffered, one barrier per chunk) and the wavefronts read their fragments
// column-wise from there: one element per lane and row, which costs LDS
// instructions but no bank conflicts (row strides put the two lane groups of
// a fragment on different banks).  The output tile is 128 x 256: four kf-tiles
// by two n-tiles per wavefront, 128 accumulator registers.  Rows are split
// into slabs over the grid; each slab writes its partial tile, summed below.

constexpr int kDwKf = 128, kDwN = 256;

template <typename T>
struct DwShape;
template <>
struct DwShape<float> {
    static constexpr int kRows = 16;          // rows per chunk
    static constexpr int kXs = kDwKf + 32;    // LDS row strides in elements: consecutive rows
    static constexpr int kDs = kDwN + 32;     // (the two lane groups) 32 banks apart
    static constexpr int kVec = 4;            // elements per 16 bytes
};
template <>
struct DwShape<bf16_t> {
    static constexpr int kRows = 32;
    static constexpr int kXs = kDwKf + 8;     // rows 8 apart (the two lane groups) 32 banks apart
    static constexpr int kDs = kDwN + 8;
    static constexpr int kVec = 8;
};

template <typename T, bool FUSE>
__global__ __launch_bounds__(256) void k_dw(const T* __restrict__ X, const T* __restrict__ dZ, RowsOp op,
                                            float* __restrict__ partial, int64_t M, int K, int N,
                                            int64_t rows_per_slab)
{
    using S = DwShape<T>;
    constexpr bool BF = sizeof(T) == 2;
    constexpr int kXUnits = S::kRows * kDwKf / S::kVec / 256;   // 16-byte units per thread and chunk
    constexpr int kDUnits = S::kRows * kDwN / S::kVec / 256;
    __shared__ __attribute__((aligned(16))) T Xs[2][S::kRows][S::kXs];
    __shared__ __attribute__((aligned(16))) T Ds[2][S::kRows][S::kDs];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, gq = lane >> 5;
    const int kf0 = blockIdx.z * kDwKf, n0 = blockIdx.y * kDwN;
    const int64_t m_beg = (int64_t)blockIdx.x * rows_per_slab;
    const int64_t m_end = std::min<int64_t>(M, m_beg + rows_per_slab);

    uint4 gx[kXUnits], gd[kDUnits];
    // FUSE: the rows of dZ are formed here (see RowsOp).  A thread's units keep their column, so its
    // pieces of a_r and its heads are fixed; the row map of a chunk is read one chunk ahead of the
    // rows themselves, which keeps a single level of loads in flight.
    __shared__ __attribute__((aligned(16))) float ars[FUSE ? kDwN : 4];   // this tile's columns of a_r
    float dsv[FUSE ? kDUnits : 1];
    int hq[FUSE ? kDUnits : 1], rk0[FUSE ? kDUnits : 1], rk1[FUSE ? kDUnits : 1];
    auto fetch_rank = [&](int64_t m0) {
        if constexpr (FUSE) {
#pragma unroll
            for (int q = 0; q < kDUnits; ++q) {
                const int u = tid + 256 * q, row = u / (kDwN / S::kVec);
                const bool ok = op.rank != nullptr && m0 + row < m_end;
                rk0[q] = ok ? op.rank[m0 + row] : 0;
                rk1[q] = ok ? op.rank[m0 + row + 1] : 0;
            }
        }
    };
    if constexpr (FUSE) {
        // a piece's values four by four: the first four of every piece, then (8-value pieces) the
        // last four, so that neighbouring lanes read neighbouring 16 bytes (no bank conflicts)
        for (int f = tid; f < kDwN; f += 256) {
            const int piece = f / S::kVec, x = f % S::kVec;
            ars[(x / 4) * (kDwN / 2) + piece * 4 + (x % 4)] = (op.ds && n0 + f < N) ? op.a_r[n0 + f] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < kDUnits; ++q) {
            const int u = tid + 256 * q, col = (u % (kDwN / S::kVec)) * S::kVec;
            hq[q] = n0 + col < N ? (n0 + col) / op.D : 0;
            dsv[q] = 0.f;
        }
        fetch_rank(m_beg);
        __syncthreads();
    }
    auto fetch = [&](int64_t m0) {
#pragma unroll
        for (int q = 0; q < kXUnits; ++q) {
            const int u = tid + 256 * q, row = u / (kDwKf / S::kVec), col = (u % (kDwKf / S::kVec)) * S::kVec;
            const bool ok = m0 + row < m_end && kf0 + col < K;
            gx[q] = ok ? *reinterpret_cast<const uint4*>(X + (m0 + row) * K + kf0 + col) : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int q = 0; q < kDUnits; ++q) {
            const int u = tid + 256 * q, row = u / (kDwN / S::kVec), col = (u % (kDwN / S::kVec)) * S::kVec;
            const bool ok = m0 + row < m_end && n0 + col < N;
            if constexpr (FUSE) {
                int64_t from = m0 + row;
                bool has = ok && op.has_E;
                if (op.rank) {
                    from = rk0[q];
                    has = has && rk1[q] > rk0[q];
                }
                gd[q] = has ? *reinterpret_cast<const uint4*>(dZ + from * N + n0 + col) : make_uint4(0u, 0u, 0u, 0u);
                dsv[q] = (ok && op.ds) ? op.ds[(m0 + row) * op.H + hq[q]] : 0.f;
            } else {
                gd[q] = ok ? *reinterpret_cast<const uint4*>(dZ + (m0 + row) * N + n0 + col) : make_uint4(0u, 0u, 0u, 0u);
            }
        }
        fetch_rank(m0 + S::kRows);
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int q = 0; q < kXUnits; ++q) {
            const int u = tid + 256 * q, row = u / (kDwKf / S::kVec), col = (u % (kDwKf / S::kVec)) * S::kVec;
            *reinterpret_cast<uint4*>(&Xs[buf][row][col]) = gx[q];
        }
#pragma unroll
        for (int q = 0; q < kDUnits; ++q) {
            const int u = tid + 256 * q, row = u / (kDwN / S::kVec), col = (u % (kDwN / S::kVec)) * S::kVec;
            if constexpr (FUSE) {
                float arv[S::kVec];
#pragma unroll
                for (int x = 0; x < S::kVec; x += 4) {
                    const float4 v = *reinterpret_cast<const float4*>(ars + (x / 4) * (kDwN / 2) + (col / S::kVec) * 4);
                    arv[x] = v.x; arv[x + 1] = v.y; arv[x + 2] = v.z; arv[x + 3] = v.w;
                }
                *reinterpret_cast<uint4*>(&Ds[buf][row][col]) = fuse_piece<T>(gd[q], dsv[q], arv);
            } else
                *reinterpret_cast<uint4*>(&Ds[buf][row][col]) = gd[q];
        }
    };

    float16_t acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    if (m_beg < m_end) {
        fetch(m_beg);
        commit(0);
    }
    __syncthreads();
    int buf = 0;
    for (int64_t m0 = m_beg; m0 < m_end; m0 += S::kRows, buf ^= 1) {
        const bool more = m0 + S::kRows < m_end;
        if (more) fetch(m0 + S::kRows);
        if (BF) {
            const uint16_t(*xs)[S::kXs] = reinterpret_cast<const uint16_t(*)[S::kXs]>(Xs[buf]);
            const uint16_t(*ds)[S::kDs] = reinterpret_cast<const uint16_t(*)[S::kDs]>(Ds[buf]);
#pragma unroll
            for (int s = 0; s < S::kRows / 16; ++s) {
                const int r0 = 16 * s + 8 * gq;
                bf16x8_t a[4], b[2];
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) {
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        w[e] = (uint32_t)xs[r0 + 2 * e][32 * kt + c] | ((uint32_t)xs[r0 + 2 * e + 1][32 * kt + c] << 16);
                    a[kt] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
                }
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {
                    uint32_t w[4];
                    const int col = 64 * wave + 32 * nt + c;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        w[e] = (uint32_t)ds[r0 + 2 * e][col] | ((uint32_t)ds[r0 + 2 * e + 1][col] << 16);
                    b[nt] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
                }
#pragma unroll
                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        acc[kt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kt], b[nt], acc[kt][nt], 0, 0, 0);
            }
        } else {
            const float(*xs)[S::kXs] = reinterpret_cast<const float(*)[S::kXs]>(Xs[buf]);
            const float(*ds)[S::kDs] = reinterpret_cast<const float(*)[S::kDs]>(Ds[buf]);
#pragma unroll
            for (int s = 0; s < S::kRows / 2; ++s) {
                const int r0 = 2 * s + gq;
                float a[4], b[2];
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) a[kt] = xs[r0][32 * kt + c];
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) b[nt] = ds[r0][64 * wave + 32 * nt + c];
#pragma unroll
                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        acc[kt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kt], b[nt], acc[kt][nt], 0, 0, 0);
            }
        }
        if (more) commit(buf ^ 1);
        __syncthreads();
    }

    // lane holds column c; register r holds row 8*(r/4) + 4*(lane/32) + r%4
    float* out = partial + (int64_t)blockIdx.x * K * N;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int n = n0 + 64 * wave + 32 * nt + c;
            if (n >= N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kf = kf0 + 32 * kt + 8 * (r / 4) + 4 * gq + (r % 4);
                if (kf < K) out[(int64_t)kf * N + n] = acc[kt][nt][r];
            }
        }
}

// dW[k] += sum over slabs of partial[slab][k].  32 consecutive elements per
// workgroup, eight threads per element taking every eighth slab; the eight
// partial sums are added in a fixed order, so the result is reproducible.
__global__ __launch_bounds__(256) void k_sum_slabs(const float* __restrict__ partial, int n_slabs, int64_t count,
                                                   float* __restrict__ dW)
{
    __shared__ float part[8][32];
    const int e = threadIdx.x & 31, zl = threadIdx.x >> 5;
    for (int64_t k0 = (int64_t)blockIdx.x * 32; k0 < count; k0 += (int64_t)gridDim.x * 32) {
        const int64_t k = k0 + e;
        float s = 0.f;
        if (k < count)
            for (int z = zl; z < n_slabs; z += 8) s += partial[(int64_t)z * count + k];
        part[zl][e] = s;
        __syncthreads();
        if (zl == 0 && k < count) {
            float t = part[0][e];
#pragma unroll
            for (int j = 1; j < 8; ++j) t += part[j][e];
            dW[k] += t;
        }
        __syncthreads();
    }
}

constexpr int kMaxSlabs = 512;

int slabs_for(int64_t n, int K, int F)
{
    const int64_t tiles = (int64_t)((K + BM - 1) / BM) * ((F + BN - 1) / BN);
    int64_t want = std::max<int64_t>(1, (1024 + tiles - 1) / tiles);
    want = std::min<int64_t>(want, kMaxSlabs);
    const int64_t by_rows = std::max<int64_t>(1, n / (4 * BK));
    return (int)std::min(want, by_rows);
}

// groups of 4 consecutive elements can be moved with one access: rows start aligned
int vec_ok(const void* p, int64_t ld, int elem_bytes)
{
    return (reinterpret_cast<uintptr_t>(p) % (4 * elem_bytes) == 0) && (ld % 4 == 0);
}

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
    g.lda = K;
    g.ldb = F;
    g.ldc = F;
    g.k_slab = K;
    g.c_split = 0;
    g.vec_a = vec_ok(X, K, dtype == SAR_F32 ? 4 : 2);
    g.vec_b = vec_ok(W, F, 4);
    SkinnyPlan plan;
    const bool want_scores = a_score || a_score2;
    // With fp32 rows the scores are two more columns of the product (z_h . a_h = x . (W_h a_h)),
    // equal to the scores of the stored rows up to fp32 rounding.  With bf16 rows they are taken
    // from the STORED (rounded) rows in one pass afterwards: every later step reads those rows,
    // and a score of the unrounded sums differs from theirs by up to the storage rounding, which
    // is enough to move LeakyReLU's kink for about one edge in a thousand.
    if (want_scores && dtype == SAR_F32 && 2 * H <= 32 && plan_skinny(X, K, Z, F, K, F, dtype, 1, &plan)) {
        SkinnyArgs sk{X, K, n, W, F, 1, Z, F, K, F, plan.chunks, a_score, a_score2, score, score2, H, D,
                      plan.stage_off};
        SAR_TRY((launch_skinny<float, float, true>(sk, plan, st)));
        return SAR_OK;
    }
    if (plan_skinny(X, K, Z, F, K, F, dtype, 0, &plan)) {
        SkinnyArgs sk{X, K, n, W, F, 1, Z, F, K, F, plan.chunks, nullptr, nullptr, nullptr, nullptr, 0, 0,
                      plan.stage_off};
        if (dtype == SAR_F32)
            SAR_TRY((launch_skinny<float, float, false>(sk, plan, st)));
        else
            SAR_TRY((launch_skinny<bf16_t, bf16_t, false>(sk, plan, st)));
    } else {
        dim3 grid((unsigned)((n + BM - 1) / BM), (unsigned)((F + BN - 1) / BN), 1);
        if (dtype == SAR_F32)
            k_gemm<float, float, float, true, false><<<grid, kGemmThreads, 0, st>>>(g);
        else
            k_gemm_bf16<bf16_t, float, bf16_t, true, false, true><<<grid, kGemmThreads, 0, st>>>(g);
        SAR_LAUNCH_CHECK();
    }
    // (one pass over the stored rows; with one vector the same vector rides along twice)
    if (a_score || a_score2) {
        const float* a1 = a_score ? a_score : a_score2;
        float* s1 = a_score ? score : score2;
        const float* a2 = a_score2 ? a_score2 : a_score;
        float* s2 = a_score2 ? score2 : score;
        return sar::gat_scores2(Z, dtype, n, H, D, a1, s1, a2, s2, stream);
    }
    return SAR_OK;
}

namespace {

// Whether both products can form the rows `op` describes while they load them (k_dw and
// k_gemm_skinny with FUSE): their aligned fast paths, a piece inside one head, the stand-in row
// readable.  dZ here is the stored part E (or the stand-in when there is none).
bool rows_op_fusable(const void* X, const void* dZ, const RowsOp& op, void* dX, int dtype, int K, int F)
{
    const int elem = dtype == SAR_F32 ? 4 : 2, vec = 16 / elem;
    if (K % vec != 0 || F % vec != 0 || op.D % vec != 0 || op.H * op.D != F || op.H > 2 * kDsRegs) return false;
    if (reinterpret_cast<uintptr_t>(X) % 16 != 0 || reinterpret_cast<uintptr_t>(dZ) % 16 != 0) return false;
    if (op.ds && reinterpret_cast<uintptr_t>(op.a_r) % 16 != 0) return false;
    SkinnyPlan plan;
    if (dX && !(plan_skinny(dZ, F, dX, K, F, K, dtype, 0, &plan) && plan_takes_rows_op(plan, F, op.H, dtype)))
        return false;
    return true;
}

// The error rows of RowsOp written out (the shapes the two products cannot form on the fly):
// the same fp32 multiply-add and the same rounding as sar_gat_bwd_end's.
template <typename T>
__global__ __launch_bounds__(256) void k_rows_store(const T* __restrict__ E, RowsOp op, T* __restrict__ out,
                                                    int64_t n, int F)
{
    const int64_t total = n * F;
    for (int64_t at = (int64_t)blockIdx.x * 256 + threadIdx.x; at < total; at += (int64_t)gridDim.x * 256) {
        const int64_t i = at / F;
        const int f = (int)(at % F);
        float o = 0.f;
        if (op.has_E) {
            int64_t from = i;
            bool present = true;
            if (op.rank) {
                from = op.rank[i];
                present = op.rank[i + 1] > (int32_t)from;
            }
            if (present) {
                if constexpr (sizeof(T) == 2)
                    o = bf16_to_f32(E[from * F + f]);
                else
                    o = E[from * F + f];
            }
        }
        if (op.ds) o = fmaf(op.ds[i * op.H + f / op.D], op.a_r[f], o);
        out[at] = from_f32<T>(o);
    }
}

// op == nullptr: dZ is the stored [n,F] operand.  Otherwise dZ is the stored part of the rows
// `op` describes and both products form the rows as they load them.
int linear_bwd_impl(const void* X, const void* dZ, const RowsOp* op, const float* W, float* dW, void* dX, int dtype,
                    int64_t n, int K, int F, void* work, size_t work_bytes, hipStream_t st)
{
    if (dW) {
        const int slabs = slabs_for(n, K, F);
        const size_t need = (size_t)slabs * K * F * sizeof(float);
        SAR_CHECK_ARG(work != nullptr && work_bytes >= need, "work_bytes=%zu is below the %zu bytes required",
                      work_bytes, need);
        // dW[K,F] = X^T dZ, contraction over the n rows, split into slabs
        const int elem = dtype == SAR_F32 ? 4 : 2, vec = 16 / elem;
        if (K % vec == 0 && F % vec == 0 && reinterpret_cast<uintptr_t>(X) % 16 == 0 &&
            reinterpret_cast<uintptr_t>(dZ) % 16 == 0) {
            const int chunk = dtype == SAR_F32 ? DwShape<float>::kRows : DwShape<bf16_t>::kRows;
            const int64_t rows_per_slab = ((n + slabs - 1) / slabs + chunk - 1) / chunk * chunk;
            dim3 grid((unsigned)slabs, (unsigned)((F + kDwN - 1) / kDwN), (unsigned)((K + kDwKf - 1) / kDwKf));
            if (op && dtype == SAR_F32)
                k_dw<float, true><<<grid, 256, 0, st>>>(static_cast<const float*>(X), static_cast<const float*>(dZ),
                                                        *op, static_cast<float*>(work), n, K, F, rows_per_slab);
            else if (op)
                k_dw<bf16_t, true><<<grid, 256, 0, st>>>(static_cast<const bf16_t*>(X),
                                                         static_cast<const bf16_t*>(dZ), *op,
                                                         static_cast<float*>(work), n, K, F, rows_per_slab);
            else if (dtype == SAR_F32)
                k_dw<float, false><<<grid, 256, 0, st>>>(static_cast<const float*>(X), static_cast<const float*>(dZ),
                                                         RowsOp{}, static_cast<float*>(work), n, K, F, rows_per_slab);
            else
                k_dw<bf16_t, false><<<grid, 256, 0, st>>>(static_cast<const bf16_t*>(X),
                                                          static_cast<const bf16_t*>(dZ), RowsOp{},
                                                          static_cast<float*>(work), n, K, F, rows_per_slab);
            SAR_LAUNCH_CHECK();
        } else {
            if (op) return sar::fail(SAR_ERR_STATE, "rows formed on the fly need the aligned dW kernel");
            GemmArgs g{};
            g.A = X;
            g.B = dZ;
            g.C = work;
            g.M = K;
            g.N = F;
            g.Kd = n;
            g.lda = K;
            g.ldb = F;
            g.ldc = F;
            g.k_slab = ((n + slabs - 1) / slabs + BK - 1) / BK * BK;
            g.c_split = (int64_t)K * F;
            g.vec_a = vec_ok(X, K, elem);
            g.vec_b = vec_ok(dZ, F, elem);
            dim3 grid((unsigned)((K + BM - 1) / BM), (unsigned)((F + BN - 1) / BN), (unsigned)slabs);
            if (dtype == SAR_F32)
                k_gemm<float, float, float, false, false><<<grid, kGemmThreads, 0, st>>>(g);
            else
                k_gemm_bf16<bf16_t, bf16_t, float, false, false, false><<<grid, kGemmThreads, 0, st>>>(g);
            SAR_LAUNCH_CHECK();
        }
        const int64_t count = (int64_t)K * F;
        k_sum_slabs<<<(unsigned)std::min<int64_t>((count + 31) / 32, 8192), 256, 0, st>>>(
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
        g.lda = F;
        g.ldb = F;
        g.ldc = K;
        g.k_slab = F;
        g.c_split = 0;
        g.vec_a = vec_ok(dZ, F, dtype == SAR_F32 ? 4 : 2);
        g.vec_b = vec_ok(W, F, 4);
        SkinnyPlan plan;
        if (plan_skinny(dZ, F, dX, K, F, K, dtype, 0, &plan)) {
            // B(k = f, n = kcol) = W[kcol * F + f]
            SkinnyArgs sk{dZ, F, n, W, 1, F, dX, K, F, K, plan.chunks, nullptr, nullptr, nullptr, nullptr, 0, 0,
                          plan.stage_off};
            if (op) {
                sk.op = *op;
                if (dtype == SAR_F32)
                    SAR_TRY((launch_skinny<float, float, false, true>(sk, plan, st)));
                else
                    SAR_TRY((launch_skinny<bf16_t, bf16_t, false, true>(sk, plan, st)));
            } else if (dtype == SAR_F32) {
                SAR_TRY((launch_skinny<float, float, false>(sk, plan, st)));
            } else {
                SAR_TRY((launch_skinny<bf16_t, bf16_t, false>(sk, plan, st)));
            }
        } else {
            if (op) return sar::fail(SAR_ERR_STATE, "rows formed on the fly need the skinny dX kernel");
            dim3 grid((unsigned)((n + BM - 1) / BM), (unsigned)((K + BN - 1) / BN), 1);
            if (dtype == SAR_F32)
                k_gemm<float, float, float, true, true><<<grid, kGemmThreads, 0, st>>>(g);
            else
                k_gemm_bf16<bf16_t, float, bf16_t, true, true, true><<<grid, kGemmThreads, 0, st>>>(g);
            SAR_LAUNCH_CHECK();
        }
    }
    return SAR_OK;
}

}  // namespace

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
    if (dW) {
        const size_t need = (size_t)slabs_for(n, K, F) * K * F * sizeof(float);
        SAR_CHECK_ARG(work != nullptr && work_bytes >= need, "work_bytes=%zu is below the %zu bytes required",
                      work_bytes, need);
    }
    return linear_bwd_impl(X, dZ, nullptr, W, dW, dX, dtype, n, K, F, work, work_bytes, sar::as_stream(stream));
}

extern "C" int sar_linear_bwd_rows(const void* X, const void* E, const int32_t* E_rank, int64_t n_E,
                                   const float* ds, const float* a_r, int H, int D, const float* W, float* dW,
                                   void* dX, int dtype, int64_t n, int K, void* rows, void* work,
                                   size_t work_bytes, void* stream)
{
    if (dtype != SAR_F32 && dtype != SAR_BF16)
        return sar::fail(SAR_ERR_UNSUPPORTED, "dtype %d is neither SAR_F32 nor SAR_BF16", dtype);
    SAR_CHECK_ARG(H > 0 && D > 0, "need H > 0 and D > 0");
    const int F = H * D;
    SAR_CHECK_ARG(n >= 0 && K > 0 && n_E >= 0, "need n >= 0, K > 0, n_E >= 0");
    if (n == 0) return SAR_OK;
    SAR_CHECK_ARG(E != nullptr || E_rank != nullptr || ds != nullptr,
                  "neither stored rows E nor the term ds (x) a_r is given");
    SAR_CHECK_ARG(E != nullptr || n_E == 0, "E is null but n_E = %lld", (long long)n_E);
    SAR_CHECK_ARG(E == nullptr || E_rank != nullptr || n_E == n, "without E_rank, E has one row per node: n_E must be n");
    SAR_CHECK_ARG((ds == nullptr) == (a_r == nullptr), "ds and a_r must be given together");
    SAR_CHECK_ARG(dW == nullptr || X != nullptr, "dW needs X");
    SAR_CHECK_ARG(dX == nullptr || W != nullptr, "dX needs W");
    SAR_CHECK_ARG(rows == nullptr || (rows != E && rows != dX), "rows must not alias E or dX");
    if (dW) {
        const size_t need = (size_t)slabs_for(n, K, F) * K * F * sizeof(float);
        SAR_CHECK_ARG(work != nullptr && work_bytes >= need, "work_bytes=%zu is below the %zu bytes required",
                      work_bytes, need);
    }
    hipStream_t st = sar::as_stream(stream);
    RowsOp op{E_rank, ds, a_r, H, D, (E != nullptr && n_E > 0) ? 1 : 0};
    if (!op.has_E && !ds) {
        // no stored row and no rank-one term: E_p = 0, dW gets nothing and dX is zero
        if (dX) {
            const unsigned g0 = (unsigned)std::min<int64_t>((n * K + 255) / 256, 16384);
            RowsOp none{};
            if (dtype == SAR_F32)
                k_rows_store<float><<<g0, 256, 0, st>>>(nullptr, none, static_cast<float*>(dX), n, K);
            else
                k_rows_store<bf16_t><<<g0, 256, 0, st>>>(nullptr, none, static_cast<bf16_t*>(dX), n, K);
            SAR_LAUNCH_CHECK();
        }
        return SAR_OK;
    }
    // where no row is stored the kernels still need an address they may read a row from
    const void* stored = op.has_E ? E : static_cast<const void*>(a_r ? a_r : ds);
    if (!rows && rows_op_fusable(X, stored, op, dX, dtype, K, F))
        return linear_bwd_impl(X, stored, &op, W, dW, dX, dtype, n, K, F, work, work_bytes, st);
    if (!rows)
        return sar::fail(SAR_ERR_UNSUPPORTED,
                         "this shape (K=%d, H=%d, D=%d) cannot form the error rows inside the products: pass `rows`, "
                         "[n,F] values of scratch, and they are written out first", K, H, D);
    const unsigned grid = (unsigned)std::min<int64_t>((n * F + 255) / 256, 16384);
    if (dtype == SAR_F32)
        k_rows_store<float><<<grid, 256, 0, st>>>(static_cast<const float*>(E), op, static_cast<float*>(rows), n, F);
    else
        k_rows_store<bf16_t><<<grid, 256, 0, st>>>(static_cast<const bf16_t*>(E), op, static_cast<bf16_t*>(rows), n, F);
    SAR_LAUNCH_CHECK();
    return linear_bwd_impl(X, rows, nullptr, W, dW, dX, dtype, n, K, F, work, work_bytes, st);
}
