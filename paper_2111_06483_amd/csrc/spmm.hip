// Sum / mean aggregation of neighbour features over partition blocks
// (Eq. 2 and the accumulation loop of Alg. 1), and its case-1 backward
// (Sec. 3.2: the gradient of a sum needs no features).
//
// All kernels are row gathers bound by HBM/L2 bandwidth: one wavefront owns one
// output row, reads the listed input rows with 16-byte lane accesses (a 1 KiB
// row is one wave-wide load), keeps several of them in flight, and adds them
// in fp32 registers.  The long rows at the head of a list are shared by the four
// wavefronts of a workgroup and merged through LDS.  The grid is persistent:
// workgroups stride over the degree-ordered row list, longest rows first.
#include <algorithm>

#include "gather_common.h"
#include "sar_internal.h"

namespace {

using namespace sar;

constexpr int kU = 4;   // rows in flight per lane group

struct PtrTab {
    const void* p[SAR_MAX_BLOCKS];
};

struct SpmmArgs {
    const int32_t* indptr;    // row offsets ([n+1]); per-block, all-blocks or transposed
    const uint32_t* indices;  // column ids (tagged with the block in the all-blocks index)
    const uint32_t* rows;     // launch list, longest class first
    int64_t n_rows, n_long;
    const void* Z;            // single input (per-block calls)
    float* acc;               // fp32 accumulator rows, read-modify-write (forward per block)
    void* out;                // typed output rows (batched forward, backward)
    const int32_t* deg;       // |N(i)| for the mean, or null
    int F;                    // values per row handled by this launch
    int ld;                   // stride between rows (values)
    int tag_shift;            // all-blocks index: block = id >> tag_shift
    int mean;
    const void* res;          // batched forward: rows added to the aggregate (Eq. 2's W_res h), or null
    int act;                  //                  SAR_ACT_* applied after that
    const int32_t* out_rank;  // backward, compact errors: row of `out` that source j owns (null: j)
};

enum class Mode { kBlock, kAll, kBackward };

// Adds the rows listed in idx[beg,end) into acc.  The wavefront takes the
// 64-edge chunks chunk0, chunk0+stride, ...
template <typename T, int G, Mode M>
__device__ inline void add_rows(float (&acc)[Vec<T>::N], const SpmmArgs& a, const void* const* ztab,
                                int beg, int end, int chunk0, int stride, const LaneMap<T, G>& lm)
{
    constexpr int VEC = Vec<T>::N;
    constexpr int SLOTS = kWave / G;
    const uint32_t mask = (M == Mode::kAll) ? ((1u << a.tag_shift) - 1u) : 0xffffffffu;
    for (int cb = beg + chunk0 * kWave; cb < end; cb += stride * kWave) {
        const int cnt = min(kWave, end - cb);
        const uint32_t mine = (lm.lane < cnt) ? a.indices[cb + lm.lane] : 0u;
        for (int k0 = 0; k0 < cnt; k0 += SLOTS * kU) {
            typename Vec<T>::Raw raw[kU];
            float w[kU];
#pragma unroll
            for (int k = 0; k < kU; ++k) {
                const int ek = k0 + k * SLOTS + lm.slot;
                const uint32_t id = __shfl(mine, ek & (kWave - 1));
                const bool ok = (ek < cnt) && lm.on;
                raw[k] = Vec<T>::zero();
                w[k] = 1.f;
                if (ok) {
                    const uint32_t j = id & mask;
                    const T* base;
                    if constexpr (M == Mode::kAll)
                        base = static_cast<const T*>(ztab[id >> a.tag_shift]);
                    else
                        base = static_cast<const T*>(a.Z);
                    raw[k] = Vec<T>::load(base + (int64_t)j * a.ld + lm.gl * VEC);
                    if constexpr (M == Mode::kBackward) {
                        if (a.mean) w[k] = 1.f / (float)max(a.deg[j], 1);
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < kU; ++k) {
                float v[VEC];
                Vec<T>::unpack(raw[k], v);
#pragma unroll
                for (int x = 0; x < VEC; ++x) {
                    if constexpr (M == Mode::kBackward)
                        acc[x] = fmaf(w[k], v[x], acc[x]);
                    else
                        acc[x] += v[x];
                }
            }
        }
    }
}

template <typename T, int G>
__device__ inline void merge_slots(float (&acc)[Vec<T>::N])
{
#pragma unroll
    for (int o = G; o < kWave; o <<= 1)
#pragma unroll
        for (int x = 0; x < Vec<T>::N; ++x) acc[x] += __shfl_xor(acc[x], o);
}

template <typename T, int G, Mode M>
__device__ inline void finish_row(const float (&acc)[Vec<T>::N], const SpmmArgs& a, int i,
                                  const LaneMap<T, G>& lm)
{
    constexpr int VEC = Vec<T>::N;
    if (lm.slot != 0 || !lm.on) return;
    int64_t row = i;
    if constexpr (M == Mode::kBackward) {
        if (a.out_rank) row = a.out_rank[i];
    }
    const int64_t o = row * a.ld + lm.gl * VEC;
    if constexpr (M == Mode::kBlock) {
        float cur[VEC];
        load_f32<VEC>(a.acc + o, cur);
#pragma unroll
        for (int x = 0; x < VEC; ++x) cur[x] += acc[x];
        store_f32<VEC>(a.acc + o, cur);
    } else {
        float v[VEC];
        float sc = 1.f;
        if constexpr (M == Mode::kAll) {
            if (a.mean) sc = 1.f / (float)max(a.deg[i], 1);
        }
#pragma unroll
        for (int x = 0; x < VEC; ++x) v[x] = acc[x] * sc;
        if constexpr (M == Mode::kAll) {
            if (a.res) {
                float r[VEC];
                Vec<T>::unpack(Vec<T>::load(static_cast<const T*>(a.res) + o), r);
#pragma unroll
                for (int x = 0; x < VEC; ++x) v[x] += r[x];
            }
            if (a.act == SAR_ACT_RELU) {
#pragma unroll
                for (int x = 0; x < VEC; ++x) v[x] = fmaxf(v[x], 0.f);
            }
        }
        Vec<T>::store(static_cast<T*>(a.out) + o, v);
    }
}

template <typename T, int G, Mode M>
__global__ __launch_bounds__(kGatherThreads) void k_spmm(SpmmArgs a, PtrTab tab, int P)
{
    constexpr int VEC = Vec<T>::N;
    __shared__ const void* ztab[SAR_MAX_BLOCKS];
    __shared__ float part[kWavesPerWG][G][VEC];
    if constexpr (M == Mode::kAll) {
        if ((int)threadIdx.x < P) ztab[threadIdx.x] = tab.p[threadIdx.x];
        __syncthreads();
    }
    const LaneMap<T, G> lm(a.F, 1, a.F);
    const int wave = threadIdx.x / kWave;

    // long rows: one workgroup each
    for (int64_t r = blockIdx.x; r < a.n_long; r += gridDim.x) {
        const int i = (int)a.rows[r];
        float acc[VEC] = {};
        add_rows<T, G, M>(acc, a, ztab, a.indptr[i], a.indptr[i + 1], wave, kWavesPerWG, lm);
        merge_slots<T, G>(acc);
        if (lm.slot == 0)
#pragma unroll
            for (int x = 0; x < VEC; ++x) part[wave][lm.gl][x] = acc[x];
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int x = 0; x < VEC; ++x) {
                float t = 0.f;
                for (int w = 0; w < kWavesPerWG; ++w) t += part[w][lm.gl][x];
                acc[x] = t;
            }
            finish_row<T, G, M>(acc, a, i, lm);
        }
        __syncthreads();
    }
    // remaining rows: one wavefront each
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerWG;
    for (int64_t r = a.n_long + (int64_t)blockIdx.x * kWavesPerWG + wave; r < a.n_rows; r += n_waves) {
        const int i = (int)a.rows[r];
        float acc[VEC] = {};
        add_rows<T, G, M>(acc, a, ztab, a.indptr[i], a.indptr[i + 1], 0, 1, lm);
        merge_slots<T, G>(acc);
        finish_row<T, G, M>(acc, a, i, lm);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void k_spmm_end(const int32_t* __restrict__ deg, int mean,
                                                  const float* __restrict__ acc, const T* res, int act, T* out,
                                                  int64_t n, int F)
{
    constexpr int VEC = Vec<T>::N;
    const int64_t total = n * (F / VEC);
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < total; k += (int64_t)gridDim.x * 256) {
        const int64_t i = k / (F / VEC);
        float v[VEC];
        load_f32<VEC>(acc + k * VEC, v);
        float sc = 1.f;
        if (mean) {
            const int d = deg[i];
            sc = d > 0 ? 1.f / (float)d : 0.f;
        }
#pragma unroll
        for (int x = 0; x < VEC; ++x) v[x] *= sc;
        if (res) {
            float r[VEC];
            Vec<T>::unpack(Vec<T>::load(res + k * VEC), r);
#pragma unroll
            for (int x = 0; x < VEC; ++x) v[x] += r[x];
        }
        if (act == SAR_ACT_RELU) {
#pragma unroll
            for (int x = 0; x < VEC; ++x) v[x] = fmaxf(v[x], 0.f);
        }
        Vec<T>::store(out + k * VEC, v);
    }
}

// G = dH * act'(.) with the derivative expressed through the output h (ReLU: 1 where h > 0)
template <typename T>
__global__ __launch_bounds__(256) void k_act_bwd(const T* h, const T* dH, T* G, int64_t n_vec)
{
    constexpr int VEC = Vec<T>::N;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < n_vec; k += (int64_t)gridDim.x * 256) {
        float hv[VEC], g[VEC];
        Vec<T>::unpack(Vec<T>::load(h + k * VEC), hv);
        Vec<T>::unpack(Vec<T>::load(dH + k * VEC), g);
#pragma unroll
        for (int x = 0; x < VEC; ++x) g[x] = hv[x] > 0.f ? g[x] : 0.f;
        Vec<T>::store(G + k * VEC, g);
    }
}

// Case-1 backward over the sources of ALL blocks in one launch.  The work list holds
// (block << tag_shift) | source for every source of every block, longest first and
// the sources without an edge last (they get dZ = 0); each entry is one row of one
// block's transposed index.
struct BwdAllTabs {
    const int32_t* t_indptr[SAR_MAX_BLOCKS];
    const uint32_t* t_indices[SAR_MAX_BLOCKS];
    void* dZ[SAR_MAX_BLOCKS];
    const int32_t* rank[SAR_MAX_BLOCKS];
};

template <typename T, int G>
__global__ __launch_bounds__(kGatherThreads) void k_spmm_bwd_all(SpmmArgs a, BwdAllTabs tabs)
{
    constexpr int VEC = Vec<T>::N;
    constexpr Mode M = Mode::kBackward;
    __shared__ float part[kWavesPerWG][G][VEC];
    const LaneMap<T, G> lm(a.F, 1, a.F);
    const int wave = threadIdx.x / kWave;
    const uint32_t mask = (1u << a.tag_shift) - 1u;
    auto locate = [&](int64_t r, SpmmArgs& la) -> int {
        const uint32_t id = __builtin_amdgcn_readfirstlane(a.rows[r]);
        const uint32_t q = id >> a.tag_shift;
        la.indptr = tabs.t_indptr[q];
        la.indices = tabs.t_indices[q];
        la.out = tabs.dZ[q];
        la.out_rank = tabs.rank[q];
        return (int)(id & mask);
    };

    for (int64_t r = blockIdx.x; r < a.n_long; r += gridDim.x) {
        SpmmArgs la = a;
        const int j = locate(r, la);
        float acc[VEC] = {};
        add_rows<T, G, M>(acc, la, nullptr, la.indptr[j], la.indptr[j + 1], wave, kWavesPerWG, lm);
        merge_slots<T, G>(acc);
        if (lm.slot == 0)
#pragma unroll
            for (int x = 0; x < VEC; ++x) part[wave][lm.gl][x] = acc[x];
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int x = 0; x < VEC; ++x) {
                float t = 0.f;
                for (int w = 0; w < kWavesPerWG; ++w) t += part[w][lm.gl][x];
                acc[x] = t;
            }
            finish_row<T, G, M>(acc, la, j, lm);
        }
        __syncthreads();
    }
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerWG;
    for (int64_t r = a.n_long + (int64_t)blockIdx.x * kWavesPerWG + wave; r < a.n_rows; r += n_waves) {
        SpmmArgs la = a;
        const int j = locate(r, la);
        float acc[VEC] = {};
        add_rows<T, G, M>(acc, la, nullptr, la.indptr[j], la.indptr[j + 1], 0, 1, lm);
        merge_slots<T, G>(acc);
        finish_row<T, G, M>(acc, la, j, lm);
    }
}

// Ep[i] (+)= Eq[rank[i]] where source i of the block has a row in the compact error, else (+)= 0
template <typename T>
__global__ __launch_bounds__(256) void k_error_add(const T* __restrict__ Eq, const int32_t* __restrict__ rank,
                                                   int accumulate, T* Ep, int64_t n, int F)
{
    constexpr int VEC = Vec<T>::N;
    const int per_row = F / VEC;
    const int64_t total = n * per_row;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < total; k += (int64_t)gridDim.x * 256) {
        const int64_t i = k / per_row;
        const int c = (int)(k % per_row) * VEC;
        const int32_t r = rank[i];
        const bool has = rank[i + 1] > r;
        if (accumulate && !has) continue;
        float v[VEC];
#pragma unroll
        for (int x = 0; x < VEC; ++x) v[x] = 0.f;
        if (has) Vec<T>::unpack(Vec<T>::load(Eq + (int64_t)r * F + c), v);
        if (accumulate) {
            float e[VEC];
            Vec<T>::unpack(Vec<T>::load(Ep + i * F + c), e);
#pragma unroll
            for (int x = 0; x < VEC; ++x) v[x] += e[x];
        }
        Vec<T>::store(Ep + i * F + c, v);
    }
}

unsigned persistent_grid(int64_t n_rows, int64_t n_long)
{
    const int64_t want = n_long + (n_rows - n_long + kWavesPerWG - 1) / kWavesPerWG;
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>(want, kMaxPersistentWGs));
}

template <typename T, Mode M>
int launch_spmm(const SpmmArgs& a, const PtrTab& tab, int P, hipStream_t st)
{
    if (a.n_rows == 0) return SAR_OK;
    const unsigned grid = persistent_grid(a.n_rows, a.n_long);
    switch (lanes_for(a.F, Vec<T>::N)) {
        case 4: k_spmm<T, 4, M><<<grid, kGatherThreads, 0, st>>>(a, tab, P); break;
        case 8: k_spmm<T, 8, M><<<grid, kGatherThreads, 0, st>>>(a, tab, P); break;
        case 16: k_spmm<T, 16, M><<<grid, kGatherThreads, 0, st>>>(a, tab, P); break;
        case 32: k_spmm<T, 32, M><<<grid, kGatherThreads, 0, st>>>(a, tab, P); break;
        case 64: k_spmm<T, 64, M><<<grid, kGatherThreads, 0, st>>>(a, tab, P); break;
        default: return sar::fail(SAR_ERR_UNSUPPORTED, "row of F=%d values is wider than 1024 bytes", a.F);
    }
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

template <typename T>
int launch_spmm_bwd_all(const SpmmArgs& a, const BwdAllTabs& tabs, hipStream_t st)
{
    if (a.n_rows == 0) return SAR_OK;
    const unsigned grid = persistent_grid(a.n_rows, a.n_long);
    switch (lanes_for(a.F, Vec<T>::N)) {
        case 4: k_spmm_bwd_all<T, 4><<<grid, kGatherThreads, 0, st>>>(a, tabs); break;
        case 8: k_spmm_bwd_all<T, 8><<<grid, kGatherThreads, 0, st>>>(a, tabs); break;
        case 16: k_spmm_bwd_all<T, 16><<<grid, kGatherThreads, 0, st>>>(a, tabs); break;
        case 32: k_spmm_bwd_all<T, 32><<<grid, kGatherThreads, 0, st>>>(a, tabs); break;
        case 64: k_spmm_bwd_all<T, 64><<<grid, kGatherThreads, 0, st>>>(a, tabs); break;
        default: return sar::fail(SAR_ERR_UNSUPPORTED, "row of F=%d values is wider than 1024 bytes", a.F);
    }
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

int check_row_shape(int dtype, int F)
{
    if (dtype != SAR_F32 && dtype != SAR_BF16)
        return sar::fail(SAR_ERR_UNSUPPORTED, "dtype %d is neither SAR_F32 nor SAR_BF16", dtype);
    if (F <= 0) return sar::fail(SAR_ERR_INVALID_ARG, "F=%d must be positive", F);
    return SAR_OK;
}

// A wavefront covers 64 lane pieces of a row (1024 bytes when the row width is a whole number of
// 16-byte pieces, less when lanes have to move 8, 4 or 2 bytes); wider rows are processed as
// several launches over column ranges, each seeing its slice of every row through the row stride.
struct ColumnChunks {
    int n, width;   // launches and values per launch (the last launch may be narrower)
    size_t fb;
    int piece;      // values per lane: the largest of 16, 8, 4, 2 bytes' worth that divides F
};

ColumnChunks column_chunks(int dtype, int F)
{
    ColumnChunks c;
    c.fb = dtype == SAR_F32 ? 4 : 2;
    c.piece = piece_for(dtype == SAR_F32, F);
    c.width = 64 * c.piece;
    c.n = (F + c.width - 1) / c.width;
    return c;
}

template <typename P>
P* shift(P* p, size_t bytes)
{
    return p ? reinterpret_cast<P*>(reinterpret_cast<uintptr_t>(p) + bytes) : nullptr;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" int sar_spmm_block(const sar_blocks_t* b, int q, const void* Zq, int dtype, int F, float* acc,
                              void* stream)
{
    SAR_CHECK_ARG(b != nullptr, "handle is null");
    SAR_CHECK_ARG(q >= 0 && q < b->P, "block %d out of range [0,%d)", q, b->P);
    SAR_TRY(check_row_shape(dtype, F));
    const sar::Block& k = b->blk[q];
    if (k.n_rows == 0) return SAR_OK;
    SAR_CHECK_ARG(Zq && acc, "Zq or acc is null");
    SAR_CHECK_ARG(aligned16(Zq) && aligned16(acc), "Zq and acc must be 16-byte aligned");
    SpmmArgs a{};
    a.indptr = k.indptr;
    a.indices = reinterpret_cast<const uint32_t*>(k.indices);
    a.rows = reinterpret_cast<const uint32_t*>(k.rows);
    a.n_rows = k.n_rows;
    a.n_long = k.n_long;
    a.ld = F;
    PtrTab tab{};
    const ColumnChunks cc = column_chunks(dtype, F);
    for (int c = 0; c < cc.n; ++c) {
        const size_t f0 = (size_t)c * cc.width;
        a.Z = shift(Zq, f0 * cc.fb);
        a.acc = acc + f0;
        a.F = std::min<int>(cc.width, F - (int)f0);
        SAR_DISPATCH_ROW(dtype, cc.piece, SAR_TRY((launch_spmm<T, Mode::kBlock>(a, tab, 0, sar::as_stream(stream)))));
    }
    return SAR_OK;
}

namespace {

int check_act(int act)
{
    if (act != SAR_ACT_NONE && act != SAR_ACT_RELU)
        return sar::fail(SAR_ERR_UNSUPPORTED, "act %d is neither SAR_ACT_NONE nor SAR_ACT_RELU", act);
    return SAR_OK;
}

}  // namespace

extern "C" int sar_act_bwd(const void* h, const void* dH, int act, void* G, int dtype, int64_t count, void* stream)
{
    if (dtype != SAR_F32 && dtype != SAR_BF16)
        return sar::fail(SAR_ERR_UNSUPPORTED, "dtype %d is neither SAR_F32 nor SAR_BF16", dtype);
    SAR_TRY(check_act(act));
    SAR_CHECK_ARG(count >= 0, "count=%lld is negative", (long long)count);
    if (count == 0) return SAR_OK;
    const int vec = piece_for(dtype == SAR_F32, (int)(count % 64 == 0 ? 64 : count % 64));
    SAR_CHECK_ARG(h && dH && G, "h, dH or G is null");
    SAR_CHECK_ARG(aligned16(h) && aligned16(dH) && aligned16(G), "h, dH and G must be 16-byte aligned");
    hipStream_t st = sar::as_stream(stream);
    if (act == SAR_ACT_NONE) {
        if (G != dH) SAR_HIP(hipMemcpyAsync(G, dH, (size_t)count * (dtype == SAR_F32 ? 4 : 2), hipMemcpyDeviceToDevice, st));
        return SAR_OK;
    }
    const int64_t n_vec = count / vec;
    const unsigned grid = (unsigned)std::min<int64_t>((n_vec + 255) / 256, 1 << 20);
    SAR_DISPATCH_ROW(dtype, vec, (k_act_bwd<T><<<grid, 256, 0, st>>>(static_cast<const T*>(h), static_cast<const T*>(dH),
                                                                     static_cast<T*>(G), n_vec)));
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

extern "C" int sar_spmm_end(const int32_t* deg, int mean, const float* acc, const void* residual, int act,
                            void* out, int dtype, int64_t n_dst, int F, void* stream)
{
    SAR_TRY(check_row_shape(dtype, F));
    SAR_TRY(check_act(act));
    SAR_CHECK_ARG(aligned16(residual), "residual must be 16-byte aligned");
    SAR_CHECK_ARG(n_dst >= 0, "n_dst is negative");
    if (n_dst == 0) return SAR_OK;
    SAR_CHECK_ARG(acc && out && (!mean || deg), "acc, out or deg is null");
    SAR_CHECK_ARG(aligned16(acc) && aligned16(out), "acc and out must be 16-byte aligned");
    const int vec = piece_for(dtype == SAR_F32, F);
    const unsigned grid = (unsigned)std::min<int64_t>((n_dst * (F / vec) + 255) / 256, 1 << 20);
    SAR_DISPATCH_ROW(dtype, vec, (k_spmm_end<T><<<grid, 256, 0, sar::as_stream(stream)>>>(
                                     deg, mean, acc, static_cast<const T*>(residual), act, static_cast<T*>(out), n_dst, F)));
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

extern "C" int sar_spmm_all(const sar_blocks_t* b, const void* const* Zq, int dtype, int F, int mean,
                            const void* residual, int act, void* out, void* stream)
{
    SAR_CHECK_ARG(b != nullptr, "handle is null");
    SAR_TRY(check_row_shape(dtype, F));
    SAR_TRY(check_act(act));
    SAR_CHECK_ARG(aligned16(residual), "residual must be 16-byte aligned");
    if (!b->f_indptr) return sar::fail(SAR_ERR_STATE, "handle was built without SAR_BUILD_FUSED");
    if (b->n_dst == 0) return SAR_OK;
    SAR_CHECK_ARG(Zq && out, "Zq or out is null");
    SAR_CHECK_ARG(aligned16(out), "out must be 16-byte aligned");
    for (int q = 0; q < b->P; ++q) {
        SAR_CHECK_ARG(Zq[q] != nullptr || b->blk[q].nnz == 0, "Zq[%d] is null", q);
        SAR_CHECK_ARG(aligned16(Zq[q]), "Zq[%d] must be 16-byte aligned", q);
    }
    hipStream_t st = sar::as_stream(stream);
    SpmmArgs a{};
    a.indptr = b->f_indptr;
    a.indices = b->f_indices;
    a.rows = reinterpret_cast<const uint32_t*>(b->f_rows);
    a.n_rows = b->n_dst;   // destinations without in-edges come last in the list and get 0
    a.n_long = b->n_f_long;
    a.deg = b->deg;
    a.ld = F;
    a.tag_shift = b->tag_shift;
    a.mean = mean;
    const ColumnChunks cc = column_chunks(dtype, F);
    for (int c = 0; c < cc.n; ++c) {
        const size_t f0 = (size_t)c * cc.width;
        PtrTab tab{};
        for (int q = 0; q < b->P; ++q) tab.p[q] = shift(Zq[q], f0 * cc.fb);
        a.out = shift(out, f0 * cc.fb);
        a.res = residual ? shift(residual, f0 * cc.fb) : nullptr;
        a.act = act;
        a.F = std::min<int>(cc.width, F - (int)f0);
        SAR_DISPATCH_ROW(dtype, cc.piece, SAR_TRY((launch_spmm<T, Mode::kAll>(a, tab, b->P, st))));
    }
    return SAR_OK;
}

extern "C" int sar_spmm_bwd_block(const sar_blocks_t* b, int q, const void* G, int mean, int dtype, int F,
                                  void* dZq, void* stream)
{
    SAR_CHECK_ARG(b != nullptr, "handle is null");
    SAR_CHECK_ARG(q >= 0 && q < b->P, "block %d out of range [0,%d)", q, b->P);
    SAR_TRY(check_row_shape(dtype, F));
    const sar::Block& k = b->blk[q];
    if (!k.t_indptr) return sar::fail(SAR_ERR_STATE, "handle was built without SAR_BUILD_TRANSPOSE");
    if (k.n_src == 0 || (sar::skips_untouched(b->flags) && k.n_t_rows == 0)) return SAR_OK;
    SAR_CHECK_ARG((G || b->n_dst == 0) && dZq, "G or dZq is null");
    SAR_CHECK_ARG(aligned16(G) && aligned16(dZq), "G and dZq must be 16-byte aligned");
    hipStream_t st = sar::as_stream(stream);
    SpmmArgs a{};
    a.indptr = k.t_indptr;
    a.indices = reinterpret_cast<const uint32_t*>(k.t_indices);
    a.rows = reinterpret_cast<const uint32_t*>(k.t_rows);
    // sources without edges come last in the list and get 0, unless the handle skips them
    a.n_rows = sar::skips_untouched(b->flags) ? k.n_t_rows : k.n_src;
    a.out_rank = (b->flags & SAR_BUILD_COMPACT) ? k.t_rank : nullptr;
    a.n_long = k.n_t_long;
    a.deg = b->deg;
    a.ld = F;
    a.mean = mean;
    PtrTab tab{};
    const ColumnChunks cc = column_chunks(dtype, F);
    for (int c = 0; c < cc.n; ++c) {
        const size_t f0 = (size_t)c * cc.width;
        a.Z = shift(G, f0 * cc.fb);
        a.out = shift(dZq, f0 * cc.fb);
        a.F = std::min<int>(cc.width, F - (int)f0);
        SAR_DISPATCH_ROW(dtype, cc.piece, SAR_TRY((launch_spmm<T, Mode::kBackward>(a, tab, 0, st))));
    }
    return SAR_OK;
}

extern "C" int sar_spmm_bwd_all(const sar_blocks_t* b, const void* G, int mean, int dtype, int F,
                                void* const* dZq, void* stream)
{
    SAR_CHECK_ARG(b != nullptr, "handle is null");
    SAR_TRY(check_row_shape(dtype, F));
    if (!b->ft_rows) return sar::fail(SAR_ERR_STATE, "handle was built without SAR_BUILD_TRANSPOSE");
    if (b->P > SAR_MAX_BLOCKS)
        return sar::fail(SAR_ERR_UNSUPPORTED, "an all-blocks call takes at most %d blocks, the handle has %d: use the "
                         "per-block calls", SAR_MAX_BLOCKS, b->P);
    int64_t n_src_total = 0;
    for (int q = 0; q < b->P; ++q) n_src_total += b->blk[q].n_src;
    if (n_src_total == 0) return SAR_OK;
    SAR_CHECK_ARG((G || b->n_dst == 0) && dZq, "G or dZq is null");
    SAR_CHECK_ARG(aligned16(G), "G must be 16-byte aligned");
    for (int q = 0; q < b->P; ++q) {
        if (b->blk[q].n_src == 0 || (sar::skips_untouched(b->flags) && b->blk[q].n_t_rows == 0)) continue;
        SAR_CHECK_ARG(dZq[q] && aligned16(dZq[q]), "dZq[%d] is null or not 16-byte aligned", q);
    }
    hipStream_t st = sar::as_stream(stream);
    SpmmArgs a{};
    a.rows = b->ft_rows;
    a.n_rows = sar::skips_untouched(b->flags) ? b->n_ft_rows : n_src_total;
    a.n_long = b->n_ft_long;
    a.deg = b->deg;
    a.ld = F;
    a.mean = mean;
    a.tag_shift = b->tag_shift;
    const ColumnChunks cc = column_chunks(dtype, F);
    for (int c = 0; c < cc.n; ++c) {
        const size_t f0 = (size_t)c * cc.width;
        BwdAllTabs tabs{};
        for (int q = 0; q < b->P; ++q) {
            const sar::Block& k = b->blk[q];
            if (k.n_src == 0) continue;
            tabs.t_indptr[q] = k.t_indptr;
            tabs.t_indices[q] = reinterpret_cast<const uint32_t*>(k.t_indices);
            tabs.dZ[q] = shift(dZq[q], f0 * cc.fb);
            tabs.rank[q] = (b->flags & SAR_BUILD_COMPACT) ? k.t_rank : nullptr;
        }
        a.Z = shift(G, f0 * cc.fb);
        a.F = std::min<int>(cc.width, F - (int)f0);
        SAR_DISPATCH_ROW(dtype, cc.piece, SAR_TRY(launch_spmm_bwd_all<T>(a, tabs, st)));
    }
    return SAR_OK;
}

extern "C" int sar_error_add(const void* Eq, const int32_t* t_rank, int accumulate, void* Ep, int dtype, int64_t n,
                             int F, void* stream)
{
    SAR_TRY(check_row_shape(dtype, F));
    SAR_CHECK_ARG(n >= 0, "n is negative");
    if (n == 0) return SAR_OK;
    SAR_CHECK_ARG(t_rank && Ep, "t_rank or Ep is null");
    SAR_CHECK_ARG(aligned16(Eq) && aligned16(Ep), "Eq and Ep must be 16-byte aligned");
    SAR_CHECK_ARG(Eq != Ep, "Eq and Ep must not alias");
    const int vec = piece_for(dtype == SAR_F32, F);
    const int64_t total = n * (F / vec);
    const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((total + 255) / 256, kMaxPersistentWGs * 4));
    hipStream_t st = sar::as_stream(stream);
    SAR_DISPATCH_ROW(dtype, vec, (k_error_add<T><<<grid, 256, 0, st>>>(static_cast<const T*>(Eq), t_rank, accumulate,
                                                                       static_cast<T*>(Ep), n, F)));
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}
