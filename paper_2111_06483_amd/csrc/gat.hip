// Fused, rematerialising attention kernels for GAT (Eq. 3; Sec. 3.3) with the
// running-maximum incremental softmax of Sec. 3.4, as row gathers on gfx950.
//
// Forward: one wavefront owns one destination row.  Per edge it reads the
// source's score half t_j and the source row z_j (16 bytes per lane, a 1 KiB
// row is one wave-wide load, several in flight), forms e = LeakyReLU(s_i+t_j)
// and folds exp(e - m) z_j into fp32 registers, rescaling when the running
// maximum m grows.  Nothing per edge is written to memory.
//
// Backward: the same gather, run over the source-major index: one wavefront
// owns one SOURCE row j, keeps z_j and t_j in registers, and for every
// destination i of j reads G_i and the per-destination record (s_i, L_i,
// delta_i), recomputes alpha = exp(e - L_i) and accumulates
// dZ_j += alpha G_i, dt_j += du in registers.  dZ_q is written once per row,
// coalesced, with no atomics; only the tiny ds[i,h] += du uses atomics.
//
// All exponentials are taken in base 2: scores are pre-multiplied by log2(e)
// (LeakyReLU commutes with a positive scale), so e2 = LeakyReLU(s2 + t2) and
// exp(e - m) = exp2(e2 - m2).
#include <algorithm>
#include <mutex>
#include <vector>

#include "gather_common.h"
#include "gat_f256.h"
#include "sar_internal.h"

namespace {

using namespace sar;

constexpr int kU = 4;   // edges in flight per lane group

struct PtrTab {
    const void* p[SAR_MAX_BLOCKS];
};

__device__ inline float leaky(float u, float slope) { return u > 0.f ? u : slope * u; }

// ------------------------------------------------------------------ forward

struct FwdArgs {
    const int32_t* indptr;
    const uint32_t* indices;
    const uint32_t* rows;
    int64_t n_rows, n_long;
    const void* Z;       // per-block call: this block's source rows
    const float* t;      //                 and their score halves [n_src,H]; null: formed from a_l
    const float* a_l;    // [H,D], used only when the source score halves are not given
    const float* s;      // destination score halves [n_dst,H]
    float* m;            // running state (per-block calls), natural-log units
    float* l;
    float* acc;
    void* out;           // batched call: normalised output rows
    float* L;            //               and log-sum-exp [n_dst,H]
    int H, D, F;         // heads, head width and row width handled by this launch
    int ldz, ldh;        // strides between nodes of the feature rows / of the per-head arrays
    int tag_shift;
    float slope;
    int act;             // SAR_ACT_*: the non-linearity of Eq. 3 on the normalised rows (batched call)
};

template <int VEC>
struct SoftState {
    float m2;          // running maximum of e, in log2 units
    float l;           // running sum of exp(e - m)
    float acc[VEC];    // running sum of exp(e - m) z
};

template <int VEC>
__device__ inline void state_reset(SoftState<VEC>& st)
{
    st.m2 = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int x = 0; x < VEC; ++x) st.acc[x] = 0.f;
}

// st <- st (+) other : the recursive aggregation property of Sec. 3.2 for the
// (max, denominator, numerator) triple.
template <int VEC>
__device__ inline void state_merge(SoftState<VEC>& st, float om2, float ol, const float (&oacc)[VEC])
{
    const float mn = fmaxf(st.m2, om2);
    const float ref = (mn == -INFINITY) ? 0.f : mn;
    const float ca = fast_exp2(st.m2 - ref), cb = fast_exp2(om2 - ref);
    st.l = st.l * ca + ol * cb;
#pragma unroll
    for (int x = 0; x < VEC; ++x) st.acc[x] = st.acc[x] * ca + oacc[x] * cb;
    st.m2 = mn;
}

// Folds the edges idx[beg,end) into st; this wavefront takes the 64-edge
// chunks chunk0, chunk0+stride, ...  s2 is the destination score half of this
// lane's head in log2 units.
template <typename T, int G, bool ALL>
__device__ inline void fwd_edges(SoftState<Vec<T>::N>& st, const FwdArgs& a, const void* const* ztab,
                                 const float* const* ttab, int beg, int end, int chunk0, int stride,
                                 const LaneMap<T, G>& lm, float s2, const float (&al)[Vec<T>::N], bool fly,
                                 bool pow2)
{
    constexpr int VEC = Vec<T>::N;
    constexpr int SLOTS = kWave / G;
    const uint32_t mask = ALL ? ((1u << a.tag_shift) - 1u) : 0xffffffffu;
    for (int cb = beg + chunk0 * kWave; cb < end; cb += stride * kWave) {
        const int cnt = min(kWave, end - cb);
        const uint32_t mine = (lm.lane < cnt) ? a.indices[cb + lm.lane] : 0u;
        for (int k0 = 0; k0 < cnt; k0 += SLOTS * kU) {
            typename Vec<T>::Raw raw[kU];
            float e2[kU];
            bool ok[kU];
#pragma unroll
            for (int k = 0; k < kU; ++k) {
                const int ek = k0 + k * SLOTS + lm.slot;
                const uint32_t id = __shfl(mine, ek & (kWave - 1));
                raw[k] = Vec<T>::zero();
                e2[k] = 0.f;
                ok[k] = ek < cnt;
                if (ek < cnt) {
                    const uint32_t j = id & mask;
                    const T* zb;
                    const float* tb;
                    if constexpr (ALL) {
                        zb = static_cast<const T*>(ztab[id >> a.tag_shift]);
                        tb = ttab[id >> a.tag_shift];
                    } else {
                        zb = static_cast<const T*>(a.Z);
                        tb = a.t;
                    }
                    if (!fly) e2[k] = tb[(int64_t)j * a.ldh + lm.h];
                    if (lm.on) raw[k] = Vec<T>::load(zb + (int64_t)j * a.ldz + lm.gl * VEC);
                }
            }
            if (fly) {   // t_j = <a_l, z_j> from the row just gathered
#pragma unroll
                for (int k = 0; k < kU; ++k) {
                    float v[VEC];
                    Vec<T>::unpack(raw[k], v);
                    float c = 0.f;
#pragma unroll
                    for (int x = 0; x < VEC; ++x) c = fmaf(al[x], v[x], c);
                    e2[k] = pow2 ? group_sum_pow2(c, lm.lph) : group_sum_any(c, lm.head_first, lm.lph);
                }
            }
            float mx = st.m2;
#pragma unroll
            for (int k = 0; k < kU; ++k) {
                // -inf marks an absent edge
                e2[k] = ok[k] ? leaky(fmaf(e2[k], kLog2e, s2), a.slope) : -INFINITY;
                mx = fmaxf(mx, e2[k]);
            }
            if (mx > st.m2) {
                const float c = fast_exp2(st.m2 - mx);   // st.m2 = -inf gives 0
                st.l *= c;
#pragma unroll
                for (int x = 0; x < VEC; ++x) st.acc[x] *= c;
                st.m2 = mx;
            }
            const float ref = (st.m2 == -INFINITY) ? 0.f : st.m2;
#pragma unroll
            for (int k = 0; k < kU; ++k) {
                const float p = fast_exp2(e2[k] - ref);
                float v[VEC];
                Vec<T>::unpack(raw[k], v);
                st.l += p;
#pragma unroll
                for (int x = 0; x < VEC; ++x) st.acc[x] = fmaf(p, v[x], st.acc[x]);
            }
        }
    }
}

template <typename T, int G>
__device__ inline void fwd_merge_slots(SoftState<Vec<T>::N>& st)
{
    constexpr int VEC = Vec<T>::N;
#pragma unroll
    for (int o = G; o < kWave; o <<= 1) {
        const float om2 = __shfl_xor(st.m2, o), ol = __shfl_xor(st.l, o);
        float oacc[VEC];
#pragma unroll
        for (int x = 0; x < VEC; ++x) oacc[x] = __shfl_xor(st.acc[x], o);
        state_merge<VEC>(st, om2, ol, oacc);
    }
}

template <typename T, int G, bool ALL, bool RELU>
__device__ inline void fwd_finish_row(SoftState<Vec<T>::N>& st, const FwdArgs& a, int i,
                                      const LaneMap<T, G>& lm)
{
    constexpr int VEC = Vec<T>::N;
    if (lm.slot != 0 || !lm.on) return;
    const int64_t o = (int64_t)i * a.ldz + lm.gl * VEC;
    if constexpr (ALL) {
        // the division by the normaliser (Sec. 3.2), and L = m + log l for the backward pass
        const float inv = st.l > 0.f ? 1.f / st.l : 0.f;
        float v[VEC];
        // the non-linearity is a template parameter: reading it from the arguments here, branch
        // or select, costs the gather loop above a fifth of its speed (measured on 2 x 100 rows)
#pragma unroll
        for (int x = 0; x < VEC; ++x) {
            v[x] = st.acc[x] * inv;
            if (RELU) v[x] = fmaxf(v[x], 0.f);
        }
        Vec<T>::store(static_cast<T*>(a.out) + o, v);
        if ((lm.gl % lm.lph) == 0)
            a.L[(int64_t)i * a.ldh + lm.h] = st.l > 0.f ? (st.m2 + fast_log2(st.l)) * kLn2 : -INFINITY;
    } else {
        store_f32<VEC>(a.acc + o, st.acc);
        if ((lm.gl % lm.lph) == 0) {
            a.m[(int64_t)i * a.ldh + lm.h] = st.m2 * kLn2;
            a.l[(int64_t)i * a.ldh + lm.h] = st.l;
        }
    }
}

template <typename T, int G, bool ALL, bool RELU>
__global__ __launch_bounds__(kGatherThreads) void k_gat_fwd(FwdArgs a, PtrTab ztab_arg, PtrTab ttab_arg,
                                                            int P)
{
    constexpr int VEC = Vec<T>::N;
    __shared__ const void* ztab[SAR_MAX_BLOCKS];
    __shared__ const float* ttab[SAR_MAX_BLOCKS];
    __shared__ float part_acc[kWavesPerWG][G][VEC];
    __shared__ float part_ml[kWavesPerWG][G][2];
    if constexpr (ALL) {
        if ((int)threadIdx.x < P) {
            ztab[threadIdx.x] = ztab_arg.p[threadIdx.x];
            ttab[threadIdx.x] = static_cast<const float*>(ttab_arg.p[threadIdx.x]);
        }
        __syncthreads();
    }
    const LaneMap<T, G> lm(a.F, a.H, a.D);
    const int wave = threadIdx.x / kWave;
    const bool fly = a.a_l != nullptr, pow2 = is_pow2(lm.lph);
    float al[VEC];
#pragma unroll
    for (int x = 0; x < VEC; ++x) al[x] = (fly && lm.on) ? a.a_l[lm.gl * VEC + x] : 0.f;

    auto load_state = [&](SoftState<VEC>& st, int i) {
        state_reset<VEC>(st);
        if constexpr (!ALL) {
            // the state carried from the previous blocks enters through lane group 0
            if (lm.slot == 0) {
                st.m2 = a.m[(int64_t)i * a.ldh + lm.h] * kLog2e;
                st.l = a.l[(int64_t)i * a.ldh + lm.h];
                if (lm.on) load_f32<VEC>(a.acc + (int64_t)i * a.ldz + lm.gl * VEC, st.acc);
            }
        }
    };

    for (int64_t r = blockIdx.x; r < a.n_long; r += gridDim.x) {
        const int i = (int)a.rows[r];
        const float s2 = a.s[(int64_t)i * a.ldh + lm.h] * kLog2e;
        SoftState<VEC> st;
        if (wave == 0)
            load_state(st, i);
        else
            state_reset<VEC>(st);
        fwd_edges<T, G, ALL>(st, a, ztab, ttab, a.indptr[i], a.indptr[i + 1], wave, kWavesPerWG, lm, s2, al, fly, pow2);
        fwd_merge_slots<T, G>(st);
        if (lm.slot == 0) {
#pragma unroll
            for (int x = 0; x < VEC; ++x) part_acc[wave][lm.gl][x] = st.acc[x];
            part_ml[wave][lm.gl][0] = st.m2;
            part_ml[wave][lm.gl][1] = st.l;
        }
        __syncthreads();
        if (wave == 0) {
            for (int w = 1; w < kWavesPerWG; ++w) {
                float oacc[VEC];
#pragma unroll
                for (int x = 0; x < VEC; ++x) oacc[x] = part_acc[w][lm.gl][x];
                state_merge<VEC>(st, part_ml[w][lm.gl][0], part_ml[w][lm.gl][1], oacc);
            }
            fwd_finish_row<T, G, ALL, RELU>(st, a, i, lm);
        }
        __syncthreads();
    }
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerWG;
    for (int64_t r = a.n_long + (int64_t)blockIdx.x * kWavesPerWG + wave; r < a.n_rows; r += n_waves) {
        const int i = (int)a.rows[r];
        const float s2 = a.s[(int64_t)i * a.ldh + lm.h] * kLog2e;
        SoftState<VEC> st;
        load_state(st, i);
        fwd_edges<T, G, ALL>(st, a, ztab, ttab, a.indptr[i], a.indptr[i + 1], 0, 1, lm, s2, al, fly, pow2);
        fwd_merge_slots<T, G>(st);
        fwd_finish_row<T, G, ALL, RELU>(st, a, i, lm);
    }
}

// ----------------------------------------------------------------- backward

struct BwdArgs {
    const int32_t* t_indptr[SAR_MAX_BLOCKS];   // per block (one entry for per-block calls)
    const int32_t* t_indices[SAR_MAX_BLOCKS];
    const void* Z[SAR_MAX_BLOCKS];
    const float* t[SAR_MAX_BLOCKS];
    void* dZ[SAR_MAX_BLOCKS];
    float* dt[SAR_MAX_BLOCKS];
    const int32_t* rank[SAR_MAX_BLOCKS];       // compact outputs: row of dZ / dt of source j (null: j)
};

struct BwdScalars {
    const uint32_t* rows;       // source work list; tagged with the block when ALL
    int64_t n_rows, n_long;
    int64_t n_wide;             // list entries [n_wide, n_rows) have few edges: several sources per wavefront
    int64_t n_touched;          // list entries [n_touched, n_rows) have no edge at all
    // all-blocks calls on a handle that lists them: the n_single list entries before n_touched are
    // the sources of ONE edge, also listed destination-major (destination, tagged source, error row)
    int64_t n_single;
    const int32_t* s_dst;
    const uint32_t* s_src;
    const int32_t* s_row;
    const int64_t* n_src_host;  // host: rows of every block's dZ_q / dt_q (null: unknown)
    int n_blocks;
    const void* G;              // [n_dst,H,D]
    const float4* rec;          // [n_dst,H]: (s*log2e, L*log2e, delta, unused)
    const float* a_l;           // [H,D]
    float* ds;                  // [n_dst,H], atomically accumulated
    float* partial;             // [gridDim.x][F] per-workgroup da_l partial sums
    int H, D, F;
    int ldz, ldh;               // node strides of feature rows / per-head arrays
    int tag_shift;
    float slope;
};

template <int VEC>
struct BwdAcc {
    float dz[VEC];   // sum_i alpha G_i
    float dt;        // sum_i du   (this lane's head)
};

// Edges (destinations) idx[beg,end) of one source row.
template <typename T, int G>
__device__ inline void bwd_edges(BwdAcc<Vec<T>::N>& ac, const BwdScalars& a, const int32_t* idx, int beg,
                                 int end, int chunk0, int stride, const LaneMap<T, G>& lm,
                                 const float (&zj)[Vec<T>::N], float t2, bool pow2)
{
    constexpr int VEC = Vec<T>::N;
    constexpr int SLOTS = kWave / G;
    const T* Gp = static_cast<const T*>(a.G);
    for (int cb = beg + chunk0 * kWave; cb < end; cb += stride * kWave) {
        const int cnt = min(kWave, end - cb);
        const int mine = (lm.lane < cnt) ? idx[cb + lm.lane] : 0;
        for (int k0 = 0; k0 < cnt; k0 += SLOTS * kU) {
            typename Vec<T>::Raw raw[kU];
            float4 rec[kU];
            int dst[kU];
#pragma unroll
            for (int k = 0; k < kU; ++k) {
                const int ek = k0 + k * SLOTS + lm.slot;
                const int i = __shfl(mine, ek & (kWave - 1));
                dst[k] = (ek < cnt) ? i : -1;
                raw[k] = Vec<T>::zero();
                rec[k] = make_float4(0.f, INFINITY, 0.f, 0.f);   // L = +inf gives alpha = 0
                if (ek < cnt) {
                    rec[k] = a.rec[(int64_t)i * a.ldh + lm.h];
                    if (lm.on) raw[k] = Vec<T>::load(Gp + (int64_t)i * a.ldz + lm.gl * VEC);
                }
            }
#pragma unroll
            for (int k = 0; k < kU; ++k) {
                float g[VEC];
                Vec<T>::unpack(raw[k], g);
                float c = 0.f;
#pragma unroll
                for (int x = 0; x < VEC; ++x) c = fmaf(g[x], zj[x], c);
                c = pow2 ? group_sum_pow2(c, lm.lph) : group_sum_any(c, lm.head_first, lm.lph);
                const float u2 = rec[k].x + t2;
                const float alpha = fast_exp2(leaky(u2, a.slope) - rec[k].y);
                const float de = alpha * (c - rec[k].z);
                const float du = u2 > 0.f ? de : a.slope * de;
#pragma unroll
                for (int x = 0; x < VEC; ++x) ac.dz[x] = fmaf(alpha, g[x], ac.dz[x]);
                ac.dt += du;
                if (dst[k] >= 0 && lm.on && (lm.gl % lm.lph) == 0)
                    unsafeAtomicAdd(a.ds + (int64_t)dst[k] * a.ldh + lm.h, du);
            }
        }
    }
}

template <typename T, int G>
__device__ inline void bwd_merge_slots(BwdAcc<Vec<T>::N>& ac)
{
#pragma unroll
    for (int o = G; o < kWave; o <<= 1) {
#pragma unroll
        for (int x = 0; x < Vec<T>::N; ++x) ac.dz[x] += __shfl_xor(ac.dz[x], o);
        ac.dt += __shfl_xor(ac.dt, o);
    }
}

template <typename T, int G, bool ALL>
__global__ __launch_bounds__(kGatherThreads) void k_gat_bwd(BwdArgs tabs, BwdScalars a)
{
    constexpr int VEC = Vec<T>::N;
    __shared__ float part[kWavesPerWG][G][VEC + 1];
    const LaneMap<T, G> lm(a.F, a.H, a.D);
    const int wave = threadIdx.x / kWave;
    const bool pow2 = is_pow2(lm.lph);
    const uint32_t mask = ALL ? ((1u << a.tag_shift) - 1u) : 0xffffffffu;

    float al[VEC], dal[VEC];
#pragma unroll
    for (int x = 0; x < VEC; ++x) {
        al[x] = lm.on ? a.a_l[lm.gl * VEC + x] : 0.f;
        dal[x] = 0.f;
    }

    // Source row j of block q: z_j and t_j stay in registers for all its edges.
    auto row_inputs = [&](uint32_t id, int& q, int& j, float (&zj)[VEC], float& t2) {
        q = ALL ? (int)(id >> a.tag_shift) : 0;
        j = (int)(id & mask);
        typename Vec<T>::Raw r = Vec<T>::zero();
        if (lm.on) r = Vec<T>::load(static_cast<const T*>(tabs.Z[q]) + (int64_t)j * a.ldz + lm.gl * VEC);
        Vec<T>::unpack(r, zj);
        if (tabs.t[q]) {
            t2 = tabs.t[q][(int64_t)j * a.ldh + lm.h] * kLog2e;
        } else {
            float c = 0.f;
#pragma unroll
            for (int x = 0; x < VEC; ++x) c = fmaf(al[x], zj[x], c);
            t2 = (pow2 ? group_sum_pow2(c, lm.lph) : group_sum_any(c, lm.head_first, lm.lph)) * kLog2e;
        }
    };
    // dZ_q[j] = sum alpha G + dt a_l ; dt_q[j] = dt ; da_l += dt z_j
    auto row_outputs = [&](const BwdAcc<VEC>& ac, int q, int j, const float (&zj)[VEC], int64_t jo) {
        if (lm.slot != 0 || !lm.on) return;
        float v[VEC];
#pragma unroll
        for (int x = 0; x < VEC; ++x) {
            v[x] = fmaf(ac.dt, al[x], ac.dz[x]);
            dal[x] = fmaf(ac.dt, zj[x], dal[x]);
        }
        Vec<T>::store(static_cast<T*>(tabs.dZ[q]) + jo * a.ldz + lm.gl * VEC, v);
        if ((lm.gl % lm.lph) == 0 && tabs.dt[q]) tabs.dt[q][jo * a.ldh + lm.h] = ac.dt;
    };

    for (int64_t r = blockIdx.x; r < a.n_long; r += gridDim.x) {
        int q, j;
        float zj[VEC], t2;
        row_inputs(a.rows[r], q, j, zj, t2);
        BwdAcc<VEC> ac = {};
        bwd_edges<T, G>(ac, a, tabs.t_indices[q], tabs.t_indptr[q][j], tabs.t_indptr[q][j + 1], wave,
                        kWavesPerWG, lm, zj, t2, pow2);
        bwd_merge_slots<T, G>(ac);
        if (lm.slot == 0) {
#pragma unroll
            for (int x = 0; x < VEC; ++x) part[wave][lm.gl][x] = ac.dz[x];
            part[wave][lm.gl][VEC] = ac.dt;
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int x = 0; x <= VEC; ++x) {
                float s = 0.f;
                for (int w = 0; w < kWavesPerWG; ++w) s += part[w][lm.gl][x];
                if (x < VEC)
                    ac.dz[x] = s;
                else
                    ac.dt = s;
            }
            row_outputs(ac, q, j, zj, tabs.rank[q] ? (int64_t)tabs.rank[q][j] : (int64_t)j);
        }
        __syncthreads();
    }
    // One source per wavefront.  Most sources of a partitioned graph have a handful of edges, so
    // what a wavefront spends its time on is the chain list entry -> edge range -> indices -> rows;
    // the first two links (and the output row) of the NEXT source are read while this one is
    // processed, the list entry of the one after that as well.
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerWG;
    int64_t r = a.n_long + (int64_t)blockIdx.x * kWavesPerWG + wave;
    struct Ahead {
        uint32_t id;
        int beg, end;
        int64_t jo;
    };
    auto look_up = [&](uint32_t id) {
        Ahead m;
        m.id = id;
        const int q = ALL ? (int)(id >> a.tag_shift) : 0, j = (int)(id & mask);
        m.beg = tabs.t_indptr[q][j];
        m.end = tabs.t_indptr[q][j + 1];
        m.jo = tabs.rank[q] ? (int64_t)tabs.rank[q][j] : (int64_t)j;
        return m;
    };
    Ahead next{};
    uint32_t id_after = 0;
    if (r < a.n_rows) next = look_up(a.rows[r]);
    if (r + n_waves < a.n_rows) id_after = a.rows[r + n_waves];
    for (; r < a.n_rows; r += n_waves) {
        const Ahead cur = next;
        if (r + n_waves < a.n_rows) next = look_up(id_after);
        if (r + 2 * n_waves < a.n_rows) id_after = a.rows[r + 2 * n_waves];
        int q, j;
        float zj[VEC], t2;
        row_inputs(cur.id, q, j, zj, t2);
        BwdAcc<VEC> ac = {};
        bwd_edges<T, G>(ac, a, tabs.t_indices[q], cur.beg, cur.end, 0, 1, lm, zj, t2, pow2);
        bwd_merge_slots<T, G>(ac);
        row_outputs(ac, q, j, zj, cur.jo);
    }

    // this workgroup's share of da_l = sum_j dt_j z_j
    __syncthreads();
    if (lm.slot == 0)
#pragma unroll
        for (int x = 0; x < VEC; ++x) part[wave][lm.gl][x] = dal[x];
    __syncthreads();
    if (wave == 0 && lm.slot == 0 && lm.on) {
        float v[VEC];
#pragma unroll
        for (int x = 0; x < VEC; ++x) {
            float s = 0.f;
            for (int w = 0; w < kWavesPerWG; ++w) s += part[w][lm.gl][x];
            v[x] = s;
        }
        store_f32<VEC>(a.partial + (int64_t)blockIdx.x * a.F + lm.gl * VEC, v);
    }
}

// out[f] += sum_w partial[w][f]
__global__ __launch_bounds__(256) void k_reduce_partials(const float* __restrict__ partial, int n_part,
                                                         int F, float* __restrict__ out)
{
    __shared__ float red[256];
    const int f = blockIdx.x;
    float s = 0.f;
    for (int w = threadIdx.x; w < n_part; w += 256) s += partial[(int64_t)w * F + f];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[f] += red[0];
}

// ---------------------------------------------------------------- node-wise

// score[v,h] = <a[h], Z[v,h]>; one lane group per node.  A second vector / output pair may ride
// along (the two halves of the attention score from one pass over Z); avec2 = null: only the first.
template <typename T, int G>
__global__ __launch_bounds__(kGatherThreads) void k_scores(const T* __restrict__ Z, int64_t n, int H, int D,
                                                           int F, int ldz, int ldh,
                                                           const float* __restrict__ avec,
                                                           float* __restrict__ score,
                                                           const float* __restrict__ avec2,
                                                           float* __restrict__ score2)
{
    constexpr int VEC = Vec<T>::N;
    constexpr int SLOTS = kWave / G;
    const LaneMap<T, G> lm(F, H, D);
    const bool pow2 = is_pow2(lm.lph);
    float av[VEC], av2[VEC];
#pragma unroll
    for (int x = 0; x < VEC; ++x) {
        av[x] = lm.on ? avec[lm.gl * VEC + x] : 0.f;
        av2[x] = (lm.on && avec2) ? avec2[lm.gl * VEC + x] : 0.f;
    }
    const int64_t wave_id = ((int64_t)blockIdx.x * kGatherThreads + threadIdx.x) / kWave;
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerWG;
    for (int64_t v0 = wave_id * SLOTS; v0 < n; v0 += n_waves * SLOTS) {
        const int64_t v = v0 + lm.slot;
        float z[VEC] = {};
        if (v < n && lm.on) Vec<T>::unpack(Vec<T>::load(Z + v * ldz + lm.gl * VEC), z);
        float c = 0.f, c2 = 0.f;
#pragma unroll
        for (int x = 0; x < VEC; ++x) {
            c = fmaf(av[x], z[x], c);
            c2 = fmaf(av2[x], z[x], c2);
        }
        c = pow2 ? group_sum_pow2(c, lm.lph) : group_sum_any(c, lm.head_first, lm.lph);
        if (avec2) c2 = pow2 ? group_sum_pow2(c2, lm.lph) : group_sum_any(c2, lm.head_first, lm.lph);
        if (v < n && lm.on && (lm.gl % lm.lph) == 0) {
            score[v * ldh + lm.h] = c;
            if (avec2) score2[v * ldh + lm.h] = c2;
        }
    }
}

// The same for head widths that do not fill whole 16-byte lane pieces: one thread per
// (node, head), element-wise reads.  Scores only; the aggregation kernels do not take such rows.
template <typename T>
__global__ __launch_bounds__(256) void k_scores_any(const T* __restrict__ Z, int64_t n, int H, int D,
                                                    const float* __restrict__ avec, float* __restrict__ score,
                                                    const float* __restrict__ avec2, float* __restrict__ score2)
{
    const int64_t total = n * H;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < total; k += (int64_t)gridDim.x * 256) {
        const int h = (int)(k % H);
        const T* z = Z + k * D;
        float c = 0.f, c2 = 0.f;
        for (int d = 0; d < D; ++d) {
            float v;
            if constexpr (sizeof(T) == 2)
                v = __uint_as_float((uint32_t)z[d].bits << 16);
            else
                v = z[d];
            c = fmaf(avec[h * D + d], v, c);
            if (avec2) c2 = fmaf(avec2[h * D + d], v, c2);
        }
        score[k] = c;
        if (avec2) score2[k] = c2;
    }
}

__global__ __launch_bounds__(256) void k_fwd_begin(float* __restrict__ m, float* __restrict__ l,
                                                   float* __restrict__ acc, int64_t n_h, int64_t n_f)
{
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < n_f; k += (int64_t)gridDim.x * 256) {
        acc[k] = 0.f;
        if (k < n_h) {
            m[k] = -INFINITY;
            l[k] = 0.f;
        }
    }
}

template <typename T, int G>
__global__ __launch_bounds__(kGatherThreads) void k_fwd_end(const float* __restrict__ m,
                                                            const float* __restrict__ l,
                                                            const float* __restrict__ acc, T* __restrict__ out,
                                                            float* __restrict__ L, int64_t n, int H, int D, int F,
                                                            int ldz, int ldh, int act)
{
    constexpr int VEC = Vec<T>::N;
    constexpr int SLOTS = kWave / G;
    const LaneMap<T, G> lm(F, H, D);
    const int64_t wave_id = ((int64_t)blockIdx.x * kGatherThreads + threadIdx.x) / kWave;
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerWG;
    for (int64_t v0 = wave_id * SLOTS; v0 < n; v0 += n_waves * SLOTS) {
        const int64_t v = v0 + lm.slot;
        if (v >= n || !lm.on) continue;
        const float lv = l[v * ldh + lm.h];
        const float inv = lv > 0.f ? 1.f / lv : 0.f;
        float a[VEC];
        load_f32<VEC>(acc + v * ldz + lm.gl * VEC, a);
#pragma unroll
        for (int x = 0; x < VEC; ++x) {
            a[x] *= inv;
            if (act == SAR_ACT_RELU) a[x] = fmaxf(a[x], 0.f);
        }
        Vec<T>::store(out + v * ldz + lm.gl * VEC, a);
        if ((lm.gl % lm.lph) == 0)
            L[v * ldh + lm.h] = lv > 0.f ? m[v * ldh + lm.h] + fast_log2(lv) * kLn2 : -INFINITY;
    }
}

// rec[i,h] = (s log2e, L log2e, <G_i, out_i>, 0) and ds = 0.  With a non-linearity, `out` holds
// h = act(aggregate) and Gr the error of h: the error of the aggregate, Gr * act'(.), is formed
// here from h alone (ReLU: h > 0 exactly where the aggregate is, and there they are equal, so
// <G_i, out_i> is unchanged) and written to Gact for the block kernels to gather.
template <typename T, int G>
__global__ __launch_bounds__(kGatherThreads) void k_bwd_begin(const T* Gr, const T* __restrict__ out,
                                                              const float* __restrict__ s,
                                                              const float* __restrict__ L, float4* __restrict__ rec,
                                                              float* __restrict__ ds, int64_t n, int H, int D, int F,
                                                              int ldz, int ldh, int act, T* Gact)
{
    constexpr int VEC = Vec<T>::N;
    constexpr int SLOTS = kWave / G;
    const LaneMap<T, G> lm(F, H, D);
    const bool pow2 = is_pow2(lm.lph);
    const int64_t wave_id = ((int64_t)blockIdx.x * kGatherThreads + threadIdx.x) / kWave;
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerWG;
    for (int64_t v0 = wave_id * SLOTS; v0 < n; v0 += n_waves * SLOTS) {
        const int64_t v = v0 + lm.slot;
        float g[VEC] = {}, o[VEC] = {};
        if (v < n && lm.on) {
            Vec<T>::unpack(Vec<T>::load(Gr + v * ldz + lm.gl * VEC), g);
            Vec<T>::unpack(Vec<T>::load(out + v * ldz + lm.gl * VEC), o);
            if (act == SAR_ACT_RELU) {
#pragma unroll
                for (int x = 0; x < VEC; ++x) g[x] = o[x] > 0.f ? g[x] : 0.f;
                Vec<T>::store(Gact + v * ldz + lm.gl * VEC, g);
            }
        }
        float c = 0.f;
#pragma unroll
        for (int x = 0; x < VEC; ++x) c = fmaf(g[x], o[x], c);
        c = pow2 ? group_sum_pow2(c, lm.lph) : group_sum_any(c, lm.head_first, lm.lph);
        if (v < n && lm.on && (lm.gl % lm.lph) == 0) {
            const int64_t k = v * ldh + lm.h;
            rec[k] = make_float4(s[k] * kLog2e, L[k] * kLog2e, c, 0.f);
            ds[k] = 0.f;
        }
    }
}

// dZdst[i] = ds[i] a_r (+ dZadd[i]) ; per-workgroup partial of da_r = sum_i ds[i] Zdst[i]
template <typename T, int G>
__global__ __launch_bounds__(kGatherThreads) void k_bwd_end(const T* __restrict__ Zdst, const float* __restrict__ ds,
                                                            const float* __restrict__ a_r, const T* dZadd,
                                                            const int32_t* __restrict__ add_rank, T* dZdst,
                                                            float* __restrict__ partial, int64_t n, int H, int D,
                                                            int F, int ldz, int ldh)
{
    constexpr int VEC = Vec<T>::N;
    constexpr int SLOTS = kWave / G;
    __shared__ float part[kWavesPerWG][kWave][VEC];
    const LaneMap<T, G> lm(F, H, D);
    const int wave = threadIdx.x / kWave;
    float ar[VEC], dar[VEC];
#pragma unroll
    for (int x = 0; x < VEC; ++x) {
        ar[x] = lm.on ? a_r[lm.gl * VEC + x] : 0.f;
        dar[x] = 0.f;
    }
    const int64_t wave_id = (int64_t)blockIdx.x * kWavesPerWG + wave;
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerWG;
    for (int64_t v0 = wave_id * SLOTS; v0 < n; v0 += n_waves * SLOTS) {
        const int64_t v = v0 + lm.slot;
        if (v >= n || !lm.on) continue;
        const float d = ds[v * ldh + lm.h];
        float z[VEC], o[VEC];
        Vec<T>::unpack(Vec<T>::load(Zdst + v * ldz + lm.gl * VEC), z);
        int64_t va = v;
        bool add = dZadd != nullptr && dZdst != nullptr;
        if (add && add_rank) {
            va = add_rank[v];
            add = add_rank[v + 1] > (int32_t)va;
        }
        if (add) {
            Vec<T>::unpack(Vec<T>::load(dZadd + va * ldz + lm.gl * VEC), o);
        } else {
#pragma unroll
            for (int x = 0; x < VEC; ++x) o[x] = 0.f;
        }
#pragma unroll
        for (int x = 0; x < VEC; ++x) {
            o[x] = fmaf(d, ar[x], o[x]);
            dar[x] = fmaf(d, z[x], dar[x]);
        }
        if (dZdst) Vec<T>::store(dZdst + v * ldz + lm.gl * VEC, o);     // null: only da_r is wanted
    }
#pragma unroll
    for (int x = 0; x < VEC; ++x) part[wave][lm.lane][x] = dar[x];
    __syncthreads();
    if (wave == 0 && lm.slot == 0 && lm.on) {
        float v[VEC];
#pragma unroll
        for (int x = 0; x < VEC; ++x) {
            float s = 0.f;
            for (int w = 0; w < kWavesPerWG; ++w)
                for (int sl = 0; sl < SLOTS; ++sl) s += part[w][sl * G + lm.gl][x];
            v[x] = s;
        }
        store_f32<VEC>(partial + (int64_t)blockIdx.x * F + lm.gl * VEC, v);
    }
}

// --------------------------------------------------------------- host side

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_act(int act)
{
    if (act != SAR_ACT_NONE && act != SAR_ACT_RELU)
        return sar::fail(SAR_ERR_UNSUPPORTED, "act %d is neither SAR_ACT_NONE nor SAR_ACT_RELU", act);
    return SAR_OK;
}

int check_shape(int dtype, int H, int D)
{
    if (dtype != SAR_F32 && dtype != SAR_BF16)
        return sar::fail(SAR_ERR_UNSUPPORTED, "dtype %d is neither SAR_F32 nor SAR_BF16", dtype);
    if (H <= 0 || D <= 0) return sar::fail(SAR_ERR_INVALID_ARG, "H and D must be positive (H=%d, D=%d)", H, D);
    // a head is covered by lanes that each move the largest piece (16, 8, 4 or 2 bytes) dividing it
    const int piece = piece_for(dtype == SAR_F32, D);
    if (D / piece > 64)
        return sar::fail(SAR_ERR_UNSUPPORTED, "one head of D=%d values in pieces of %d needs more than the 64 lanes "
                         "of a wavefront", D, piece);
    return SAR_OK;
}

// Heads are independent in Eq. 3, so a layer whose rows exceed what one wavefront covers
// (64 lane pieces: 1024 bytes when the head width is a whole number of 16-byte pieces) is
// processed as several launches over groups of heads, each launch seeing its slice of every
// row through the row stride.
struct HeadGroups {
    int n, Hg, Fg;       // groups, heads per group, values per group
    size_t fb;           // bytes per feature value
    int piece;           // values per lane of the generic and node-wise kernels (divides D)
    bool fast_fwd;       // the specialised forward / backward gather kernels take a group (they use the
    bool fast_bwd;       // full row type)
    int full;            // values per lane of the full row type: 4 (fp32) or 8 (bf16)
};

// Lanes per head of the specialised kernels for head width D: the power of two >= D/4 (4..64), or 0.
int lanes_per_head(int D)
{
    if (D % 4 != 0 || D > 256) return 0;
    int lph = 4;
    while (lph * 4 < D) lph *= 2;
    return lph;
}

// The specialised kernels give every head LPH lanes of 4 values.  Exact geometry: contiguous rows
// of 256 values, LPH = D/4 (4..64), 64/LPH heads.  Padded geometry (built for LPH = 8, 16, 32, 64):
// heads of any width that is a multiple of 4 up to 4 LPH, rows of any stride, up to 64/LPH heads per
// launch; lanes a head does not need, and head groups the launch has no head for, stay idle, and a
// layer of more heads runs as several launches over groups of heads.  The gathers are bound by
// memory, not by lanes, so idle lanes cost little:
//   at least 3/8 of the 64 lanes busy: faster than the generic kernels in both passes, also over
//     several launches (4 x 32, 5.96 -> 3.8 ms per step of the products-sized share; 16 x 32 in
//     rows of 512, 19.2 -> 14.9 ms; 1 x 100, 11.5 -> 5.3 ms; 3 x 64 and 6 x 32 on 48 lanes);
//   fewer ("sparse"): only the backward pass gains, and only when the whole layer is ONE launch
//     (the generic backward gives every source a wavefront however few its edges: 4 x 16,
//     3.43 -> 1.83 ms; its forward stays ahead, 0.69 against 0.94 ms; over several launches the
//     repeated index traffic costs more than it saves).
// Lanes per head of the padded geometry for head width D, or 0.
int padded_lanes(int D)
{
    const int need = lanes_per_head(D);
    return need == 0 ? 0 : std::max(8, need);
}
// Whether a launch of Hg heads of width D would leave more than 5/8 of the lanes idle.
bool sparse_launch(int Hg, int D) { return Hg * (D / 4) * 8 < 3 * 64; }

struct FastGeo {
    int lph;     // 0: not applicable
    bool pad;
    bool sparse; // fewer than 3/8 of the lanes carry values: backward pass only
};
FastGeo fast_geo(int H, int D, int ldz);

HeadGroups head_groups(int dtype, int H, int D)
{
    HeadGroups g;
    g.fb = dtype == SAR_F32 ? 4 : 2;
    g.full = dtype == SAR_F32 ? 4 : 8;
    g.piece = piece_for(dtype == SAR_F32, D);
    int hg = std::max<int>(1, 64 * g.piece / D);
    hg = std::min(hg, H);
    while (H % hg != 0) --hg;
    // heads per launch of the specialised kernels, where they apply (see padded_lanes): the largest
    // divisor of H that fits a wavefront
    const int lph = lanes_per_head(D);
    if (lph > 0 && H * lph == 64 && H * D == f256::kF) {
        hg = H;                                   // the exact geometry: all heads in one launch
    } else if (lph > 0) {
        for (int cand = std::min(H, 64 / padded_lanes(D)); cand >= 1; --cand) {
            if (H % cand != 0) continue;
            if (!sparse_launch(cand, D) || cand == H) hg = cand;
            break;
        }
    }
    g.Hg = hg;
    g.n = H / hg;
    g.Fg = hg * D;
    const FastGeo geo = fast_geo(hg, D, H * D);
    g.fast_bwd = geo.lph != 0;
    g.fast_fwd = geo.lph != 0 && !geo.sparse;
    return g;
}

template <typename P>
P* shift(P* p, size_t bytes)
{
    return p ? reinterpret_cast<P*>(reinterpret_cast<uintptr_t>(p) + bytes) : nullptr;
}

unsigned persistent_grid(int64_t n_rows, int64_t n_long)
{
    const int64_t want = n_long + (n_rows - n_long + kWavesPerWG - 1) / kWavesPerWG;
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>(want, kMaxPersistentWGs));
}

unsigned nodewise_grid(int64_t n, int slots)
{
    const int64_t waves = (n + slots - 1) / slots;
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>((waves + kWavesPerWG - 1) / kWavesPerWG, kMaxPersistentWGs));
}

#define SAR_DISPATCH_G(T, F, CALL)                                                   \
    switch (lanes_for((F), Vec<T>::N)) {                                             \
        case 4: { constexpr int kG = 4; CALL; } break;                                \
        case 8: { constexpr int kG = 8; CALL; } break;                                \
        case 16: { constexpr int kG = 16; CALL; } break;                              \
        case 32: { constexpr int kG = 32; CALL; } break;                              \
        default: { constexpr int kG = 64; CALL; } break;                              \
    }

// Workgroups that can be resident at once for kernel `fn` (persistent grids are
// sized to this, so that every workgroup starts immediately).
template <typename Fn>
int resident_workgroups(Fn fn)
{
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return kMaxPersistentWGs;
        n_cu = prop.multiProcessorCount;
    }
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kGatherThreads, 0) != hipSuccess || per_cu <= 0)
        return kMaxPersistentWGs;
    return std::min(kMaxPersistentWGs, n_cu * per_cu);
}

unsigned persistent_grid_for(int64_t n_rows, int64_t n_long, int resident)
{
    const int64_t want = n_long + (n_rows - n_long + kWavesPerWG - 1) / kWavesPerWG;
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>(want, resident));
}

// Whether the specialised kernels take a launch of H heads of width D in rows of stride ldz, and
// in which geometry: exact (contiguous rows of 256 values, power-of-two head width) or padded
// (64/LPH heads of any width up to 4*LPH that is a multiple of 4, any row stride; built for
// LPH = 8, 16, 32, 64).  Lanes move 4 values (16 bytes of fp32, 8 bytes of bf16) either way.
FastGeo fast_geo(int H, int D, int ldz)
{
    const int lph = lanes_per_head(D);
    if (lph == 0) return FastGeo{0, false, false};
    if (H * lph == 64 && D == 4 * lph && ldz == f256::kF) return FastGeo{lph, false, false};
    const int lanes = padded_lanes(D);
    if (H < 1 || H * lanes > 64) return FastGeo{0, false, false};
    const bool sparse = sparse_launch(H, D);
    if (sparse && H * D != ldz) return FastGeo{0, false, false};   // sparse launches pay only as the single one
    return FastGeo{lanes, true, sparse};
}

template <typename T, int LPH, bool ALL, bool FLY, bool PAD>
int launch_fwd_f256(const FwdArgs& a, const PtrTab& zt, const PtrTab& tt, hipStream_t st)
{
    constexpr int B = LPH >= 8 ? 8 : 4;
    auto fn = f256::k_gat_fwd_f256<T, LPH, B, ALL, FLY, PAD>;
    static const int resident = resident_workgroups(fn);
    f256::FwdP p{};
    p.indptr = a.indptr; p.indices = a.indices; p.rows = a.rows;
    p.n_rows = a.n_rows; p.n_long = a.n_long;
    p.Z = a.Z; p.t = a.t; p.a_l = a.a_l; p.s = a.s; p.m = a.m; p.l = a.l; p.acc = a.acc; p.out = a.out; p.L = a.L;
    p.H = a.H; p.tag_shift = a.tag_shift; p.slope = a.slope; p.act = a.act;
    p.ld = a.ldz; p.ldh = a.ldh; p.D = a.D;
    f256::Tabs tabs{};
    for (int q = 0; q < SAR_MAX_BLOCKS; ++q) {
        tabs.Z[q] = zt.p[q];
        tabs.t[q] = static_cast<const float*>(tt.p[q]);
    }
    fn<<<persistent_grid_for(a.n_rows, a.n_long, resident), kGatherThreads, 0, st>>>(p, tabs);
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

template <typename T, bool ALL>
int launch_fwd(const FwdArgs& a, const PtrTab& zt, const PtrTab& tt, int P, hipStream_t st)
{
    if (a.n_rows == 0) return SAR_OK;
    if constexpr (is_full_row<T>::value) {
#define SAR_FWD_F256(LPH, PAD)                                                             \
    return a.a_l ? launch_fwd_f256<T, LPH, ALL, true, PAD>(a, zt, tt, st)                  \
                 : launch_fwd_f256<T, LPH, ALL, false, PAD>(a, zt, tt, st)
        const FastGeo geo = fast_geo(a.H, a.D, a.ldz);
        if (geo.sparse) {
            // the generic forward kernel is the faster one here
        } else if (geo.pad) {
            switch (geo.lph) {
                case 8: SAR_FWD_F256(8, true);
                case 16: SAR_FWD_F256(16, true);
                case 32: SAR_FWD_F256(32, true);
                case 64: SAR_FWD_F256(64, true);
                default: break;
            }
        } else {
            switch (geo.lph) {
                case 4: SAR_FWD_F256(4, false);
                case 8: SAR_FWD_F256(8, false);
                case 16: SAR_FWD_F256(16, false);
                case 32: SAR_FWD_F256(32, false);
                case 64: SAR_FWD_F256(64, false);
                default: break;
            }
        }
#undef SAR_FWD_F256
        if (a.D % Vec<T>::N != 0)
            return sar::fail(SAR_ERR_STATE, "head width %d reached the generic kernel with %d-value pieces", a.D, Vec<T>::N);
    }
    const unsigned grid = persistent_grid(a.n_rows, a.n_long);
    if constexpr (ALL) {
        if (a.act == SAR_ACT_RELU) {
            SAR_DISPATCH_G(T, a.F, (k_gat_fwd<T, kG, true, true><<<grid, kGatherThreads, 0, st>>>(a, zt, tt, P)));
            SAR_LAUNCH_CHECK();
            return SAR_OK;
        }
    }
    SAR_DISPATCH_G(T, a.F, (k_gat_fwd<T, kG, ALL, false><<<grid, kGatherThreads, 0, st>>>(a, zt, tt, P)));
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

// The same pair of kernels in the padded geometry.  The few-edges kernel also takes the sources
// without an edge at the end of the list (it writes their zero rows).
template <typename T, int LPH, bool ALL>
int launch_bwd_f256_padded(const BwdArgs& tabs, const BwdScalars& a, unsigned* grid_out, hipStream_t st)
{
    constexpr int B = 8;
    auto wide = f256::k_gat_bwd_f256<T, LPH, B, ALL, true>;
    auto few = f256::k_gat_bwd_few<T, LPH, ALL, true>;
    auto single = f256::k_gat_bwd_single<T, LPH, true>;
    static const int resident_wide = resident_workgroups(wide);
    static const int resident_few = resident_workgroups(few);
    static const int resident_single = resident_workgroups(single);
    f256::BwdTabs t{};
    for (int q = 0; q < SAR_MAX_BLOCKS; ++q) {
        t.t_indptr[q] = tabs.t_indptr[q]; t.t_indices[q] = tabs.t_indices[q];
        t.Z[q] = tabs.Z[q]; t.t[q] = tabs.t[q]; t.dZ[q] = tabs.dZ[q]; t.dt[q] = tabs.dt[q];
        t.rank[q] = tabs.rank[q];
    }
    f256::BwdP p{};
    p.rows = a.rows; p.n_rows = a.n_wide; p.n_long = std::min(a.n_long, a.n_wide);
    p.G = a.G; p.rec = a.rec; p.a_l = a.a_l; p.ds = a.ds; p.partial = a.partial;
    p.H = a.H; p.tag_shift = a.tag_shift; p.slope = a.slope;
    p.ld = a.ldz; p.ldh = a.ldh; p.D = a.D;
    unsigned g_wide = 0, g_few = 0, g_single = 0;
    if (a.n_wide > 0) {
        g_wide = persistent_grid_for(p.n_rows, p.n_long, resident_wide);
        wide<<<g_wide, kGatherThreads, 0, st>>>(t, p);
        SAR_LAUNCH_CHECK();
    }
    // The sources of one edge go destination-major where the handle lists them that way.  In the
    // work list they sit between the other few-edge sources and the ones without an edge, so the
    // few-edges kernel takes the list in two pieces around them.
    const int64_t n_edged = std::max(a.n_wide, std::min(a.n_rows, a.n_touched));
    const int64_t n_pulled = (ALL && a.s_dst && a.n_single <= n_edged - a.n_wide) ? a.n_single : 0;
    const int64_t per_wg = (int64_t)(B / 2) * kWavesPerWG;
    const int64_t piece[2][2] = {{a.n_wide, n_pulled ? n_edged - n_pulled : a.n_rows}, {n_edged, n_pulled ? a.n_rows : n_edged}};
    for (int k = 0; k < 2; ++k) {
        const int64_t n = piece[k][1] - piece[k][0];
        if (n <= 0) continue;
        const unsigned g = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n + per_wg - 1) / per_wg, resident_few));
        few<<<g, kGatherThreads, 0, st>>>(t, p, piece[k][0], piece[k][1], (int)(g_wide + g_few));
        SAR_LAUNCH_CHECK();
        g_few += g;
    }
    if (n_pulled > 0) {
        const f256::SingleP sp{a.s_dst, a.s_src, a.s_row, n_pulled};
        const int64_t per_wg_s = (int64_t)kWave * kWavesPerWG;
        g_single = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n_pulled + per_wg_s - 1) / per_wg_s, resident_single));
        single<<<g_single, kGatherThreads, 0, st>>>(t, p, sp, (int)(g_wide + g_few));
        SAR_LAUNCH_CHECK();
    }
    *grid_out = g_wide + g_few + g_single;
    return SAR_OK;
}

// da_l[h*D + 4k + x] += sum_w partial[w][(h*LPH + k)*4 + x]: the padded kernels leave their
// partial sums in lane order (256 slots per workgroup)
__global__ __launch_bounds__(256) void k_reduce_partials_padded(const float* __restrict__ partial, int n_part,
                                                                int lph, int H, int D, float* __restrict__ out)
{
    __shared__ float red[256];
    const int slot = blockIdx.x, lane = slot >> 2, x = slot & 3;
    const int h = lane / lph, k = lane % lph;
    if (h >= H || 4 * k >= D) return;
    float s = 0.f;
    for (int w = threadIdx.x; w < n_part; w += 256) s += partial[(int64_t)w * 256 + slot];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[h * D + 4 * k + x] += red[0];
}

// The sources without an edge in their block (the tail of the work list): their rows of dZ_q and
// dt_q are zero, and nothing has to be read for that but the list entry.
template <typename T, bool ALL>
__global__ __launch_bounds__(256) void k_bwd_zero_rows(f256::BwdTabs tabs, const uint32_t* __restrict__ rows,
                                                       int64_t r_begin, int64_t r_end, int H, int tag_shift)
{
    constexpr int kPieces = f256::kF * (int)sizeof(T) / 16;   // 16-byte pieces of a row
    __shared__ void* s_dZ[SAR_MAX_BLOCKS];
    __shared__ float* s_dt[SAR_MAX_BLOCKS];
    if (threadIdx.x < SAR_MAX_BLOCKS) {
        s_dZ[threadIdx.x] = tabs.dZ[threadIdx.x];
        s_dt[threadIdx.x] = tabs.dt[threadIdx.x];
    }
    __syncthreads();
    const uint32_t mask = ALL ? ((1u << tag_shift) - 1u) : 0xffffffffu;
    const int64_t total = (r_end - r_begin) * kPieces;
    for (int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x; p < total; p += (int64_t)gridDim.x * 256) {
        const uint32_t id = rows[r_begin + p / kPieces];
        const int piece = (int)(p % kPieces);
        const int q = ALL ? (int)(id >> tag_shift) : 0;
        const int64_t j = (int64_t)(id & mask);
        reinterpret_cast<uint4*>(static_cast<T*>(s_dZ[q]) + j * f256::kF)[piece] = make_uint4(0u, 0u, 0u, 0u);
        if (piece < H && s_dt[q]) s_dt[q][j * H + piece] = 0.f;
    }
}

__global__ __launch_bounds__(256) void k_zero_f32(float* __restrict__ p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0.f;
}

template <typename T, int LPH, bool ALL>
int launch_bwd_f256(const BwdArgs& tabs, const BwdScalars& a, unsigned* grid_out, hipStream_t st)
{
    constexpr int B = LPH >= 8 ? 8 : 4;
    auto wide = f256::k_gat_bwd_f256<T, LPH, B, ALL, false>;
    auto few = f256::k_gat_bwd_few<T, LPH, ALL, false>;
    auto single = f256::k_gat_bwd_single<T, LPH, false>;
    constexpr int kPerWave = B / 2;     // sources a wavefront of that kernel takes at once
    static const int resident_wide = resident_workgroups(wide);
    static const int resident_few = resident_workgroups(few);
    static const int resident_single = resident_workgroups(single);
    f256::BwdTabs t{};
    for (int q = 0; q < SAR_MAX_BLOCKS; ++q) {
        t.t_indptr[q] = tabs.t_indptr[q]; t.t_indices[q] = tabs.t_indices[q];
        t.Z[q] = tabs.Z[q]; t.t[q] = tabs.t[q]; t.dZ[q] = tabs.dZ[q]; t.dt[q] = tabs.dt[q];
        t.rank[q] = tabs.rank[q];
    }
    f256::BwdP p{};
    p.rows = a.rows; p.n_rows = a.n_wide; p.n_long = std::min(a.n_long, a.n_wide);
    p.G = a.G; p.rec = a.rec; p.a_l = a.a_l; p.ds = a.ds; p.partial = a.partial;
    p.H = a.H; p.tag_shift = a.tag_shift; p.slope = a.slope;
    unsigned g_wide = 0, g_few = 0, g_single = 0;
    const int64_t n_edged = std::max(a.n_wide, std::min(a.n_rows, a.n_touched));
    // the sources of one edge (the end of the edged part of the list) go destination-major where
    // the handle lists them that way
    const int64_t n_pulled = (ALL && a.s_dst && a.n_single <= n_edged - a.n_wide) ? a.n_single : 0;
    const int64_t n_few_end = n_edged - n_pulled;
    // Where many sources have no edge (a 16-way split leaves 46% of them without one), their 32-byte
    // rows of dt_q scattered through the array cost more to zero one by one than the whole array
    // does in one sweep ahead of the kernels that write the other rows.
    const bool sweep_dt = a.n_src_host != nullptr && (a.n_rows - n_edged) * 4 > a.n_rows;
    if (sweep_dt) {
        for (int q = 0; q < a.n_blocks; ++q) {
            const int64_t n = a.n_src_host[q] * a.H;
            if (n == 0 || !tabs.dt[q]) continue;
            k_zero_f32<<<(unsigned)std::min<int64_t>((n + 255) / 256, kMaxPersistentWGs), 256, 0, st>>>(tabs.dt[q], n);
            SAR_LAUNCH_CHECK();
        }
    }
    if (a.n_wide > 0) {
        // sources with at least 8 edges: one wavefront (or workgroup) each
        g_wide = persistent_grid_for(p.n_rows, p.n_long, resident_wide);
        wide<<<g_wide, kGatherThreads, 0, st>>>(t, p);
        SAR_LAUNCH_CHECK();
    }
    if (n_few_end > a.n_wide) {
        // the other sources with edges, several per wavefront
        const int64_t n = n_few_end - a.n_wide;
        const int64_t per_wg = (int64_t)kPerWave * kWavesPerWG;
        g_few = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n + per_wg - 1) / per_wg, resident_few));
        few<<<g_few, kGatherThreads, 0, st>>>(t, p, a.n_wide, n_few_end, (int)g_wide);
        SAR_LAUNCH_CHECK();
    }
    if (n_pulled > 0) {
        const f256::SingleP sp{a.s_dst, a.s_src, a.s_row, n_pulled};
        const int64_t per_wg = (int64_t)kWave * kWavesPerWG;
        g_single = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n_pulled + per_wg - 1) / per_wg, resident_single));
        single<<<g_single, kGatherThreads, 0, st>>>(t, p, sp, (int)(g_wide + g_few));
        SAR_LAUNCH_CHECK();
    }
    if (a.n_rows > n_edged) {
        const int64_t pieces = (a.n_rows - n_edged) * (f256::kF * (int64_t)sizeof(T) / 16);
        const unsigned g_zero = (unsigned)std::min<int64_t>((pieces + 255) / 256, kMaxPersistentWGs);
        k_bwd_zero_rows<T, ALL><<<g_zero, 256, 0, st>>>(t, a.rows, n_edged, a.n_rows, sweep_dt ? 0 : a.H,
                                                       a.tag_shift);
        SAR_LAUNCH_CHECK();
    }
    *grid_out = g_wide + g_few + g_single;
    return SAR_OK;
}

template <typename T, bool ALL>
int launch_bwd(const BwdArgs& tabs, BwdScalars& a, float* da_l, hipStream_t st)
{
    if (a.n_rows == 0) return SAR_OK;
    unsigned grid = persistent_grid(a.n_rows, a.n_long);
    bool done = false;
    if constexpr (is_full_row<T>::value) {
        const FastGeo geo = fast_geo(a.H, a.D, a.ldz);
        if (geo.pad) {
            switch (geo.lph) {
                case 8: SAR_TRY((launch_bwd_f256_padded<T, 8, ALL>(tabs, a, &grid, st))); break;
                case 16: SAR_TRY((launch_bwd_f256_padded<T, 16, ALL>(tabs, a, &grid, st))); break;
                case 32: SAR_TRY((launch_bwd_f256_padded<T, 32, ALL>(tabs, a, &grid, st))); break;
                default: SAR_TRY((launch_bwd_f256_padded<T, 64, ALL>(tabs, a, &grid, st))); break;
            }
            k_reduce_partials_padded<<<256, 256, 0, st>>>(a.partial, (int)grid, geo.lph, a.H, a.D, da_l);
            SAR_LAUNCH_CHECK();
            return SAR_OK;
        }
        done = true;
        switch (geo.lph) {
            case 4: SAR_TRY((launch_bwd_f256<T, 4, ALL>(tabs, a, &grid, st))); break;
            case 8: SAR_TRY((launch_bwd_f256<T, 8, ALL>(tabs, a, &grid, st))); break;
            case 16: SAR_TRY((launch_bwd_f256<T, 16, ALL>(tabs, a, &grid, st))); break;
            case 32: SAR_TRY((launch_bwd_f256<T, 32, ALL>(tabs, a, &grid, st))); break;
            case 64: SAR_TRY((launch_bwd_f256<T, 64, ALL>(tabs, a, &grid, st))); break;
            default: done = false; break;
        }
        if (!done && a.D % Vec<T>::N != 0)
            return sar::fail(SAR_ERR_STATE, "head width %d reached the generic kernel with %d-value pieces", a.D, Vec<T>::N);
    }
    if (!done) {
        SAR_DISPATCH_G(T, a.F, (k_gat_bwd<T, kG, ALL><<<grid, kGatherThreads, 0, st>>>(tabs, a)));
        SAR_LAUNCH_CHECK();
    }
    k_reduce_partials<<<a.F, 256, 0, st>>>(a.partial, (int)grid, a.F, da_l);
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

// room for one row of 256 partial sums per workgroup of the (up to) four backward launches of a call
size_t workspace_bytes(int F) { return (size_t)4 * kMaxPersistentWGs * F * sizeof(float); }

}  // namespace

// One pass over Z for one or two score vectors (a2/score2 may be null).
int sar::gat_scores2(const void* Z, int dtype, int64_t n, int H, int D, const float* a, float* score,
                     const float* a2, float* score2, void* stream)
{
    if (dtype != SAR_F32 && dtype != SAR_BF16)
        return sar::fail(SAR_ERR_UNSUPPORTED, "dtype %d is neither SAR_F32 nor SAR_BF16", dtype);
    SAR_CHECK_ARG(H > 0 && D > 0, "H and D must be positive (H=%d, D=%d)", H, D);
    SAR_CHECK_ARG((a2 == nullptr) == (score2 == nullptr), "the second vector and its output go together");
    if (D / piece_for(dtype == SAR_F32, D) > 64) {
        // a head that no wavefront covers in lane pieces (an odd width above 64, say): one thread
        // per (node, head); any width is a valid product of the transform
        SAR_CHECK_ARG(n >= 0, "n is negative");
        if (n == 0) return SAR_OK;
        SAR_CHECK_ARG(Z && a && score, "Z, a or score is null");
        const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n * H + 255) / 256, kMaxPersistentWGs * 4));
        if (dtype == SAR_F32)
            k_scores_any<float><<<grid, 256, 0, sar::as_stream(stream)>>>(static_cast<const float*>(Z), n, H, D, a,
                                                                          score, a2, score2);
        else
            k_scores_any<bf16_t><<<grid, 256, 0, sar::as_stream(stream)>>>(static_cast<const bf16_t*>(Z), n, H, D, a,
                                                                           score, a2, score2);
        SAR_LAUNCH_CHECK();
        return SAR_OK;
    }
    SAR_TRY(check_shape(dtype, H, D));
    SAR_CHECK_ARG(n >= 0, "n is negative");
    if (n == 0) return SAR_OK;
    SAR_CHECK_ARG(Z && a && score, "Z, a or score is null");
    SAR_CHECK_ARG(aligned16(Z), "Z must be 16-byte aligned");
    const int F = H * D;
    const HeadGroups hg = head_groups(dtype, H, D);
    hipStream_t st = sar::as_stream(stream);
    for (int g = 0; g < hg.n; ++g) {
        const void* Zg = shift(Z, (size_t)g * hg.Fg * hg.fb);
        const float* ag = a + (size_t)g * hg.Fg;
        float* sg = score + (size_t)g * hg.Hg;
        const float* ag2 = a2 ? a2 + (size_t)g * hg.Fg : nullptr;
        float* sg2 = score2 ? score2 + (size_t)g * hg.Hg : nullptr;
        SAR_DISPATCH_ROW(dtype, hg.piece,
                         SAR_DISPATCH_G(T, hg.Fg, (k_scores<T, kG><<<nodewise_grid(n, kWave / kG), kGatherThreads, 0, st>>>(
                                                      static_cast<const T*>(Zg), n, hg.Hg, D, hg.Fg, F, H, ag, sg, ag2, sg2))));
        SAR_LAUNCH_CHECK();
    }
    return SAR_OK;
}

extern "C" int sar_gat_scores(const void* Z, int dtype, int64_t n, int H, int D, const float* a,
                              float* score, void* stream)
{
    return sar::gat_scores2(Z, dtype, n, H, D, a, score, nullptr, nullptr, stream);
}

extern "C" int sar_gat_fwd_begin(float* m, float* l, float* acc, int64_t n_dst, int H, int D, void* stream)
{
    SAR_CHECK_ARG(n_dst >= 0 && H > 0 && D > 0, "need n_dst >= 0, H > 0, D > 0");
    if (n_dst == 0) return SAR_OK;
    SAR_CHECK_ARG(m && l && acc, "m, l or acc is null");
    const int64_t n_f = n_dst * H * D;
    const unsigned grid = (unsigned)std::min<int64_t>((n_f + 255) / 256, 1 << 20);
    k_fwd_begin<<<grid, 256, 0, sar::as_stream(stream)>>>(m, l, acc, n_dst * H, n_f);
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

extern "C" int sar_gat_fwd_block(const sar_blocks_t* b, int q, const void* Zq, const float* s,
                                 const float* tq, const float* a_l, int dtype, int H, int D, float slope,
                                 float* m, float* l, float* acc, void* stream)
{
    SAR_CHECK_ARG(b != nullptr, "handle is null");
    SAR_CHECK_ARG(q >= 0 && q < b->P, "block %d out of range [0,%d)", q, b->P);
    SAR_TRY(check_shape(dtype, H, D));
    const sar::Block& k = b->blk[q];
    if (k.n_rows == 0) return SAR_OK;
    SAR_CHECK_ARG(Zq && s && m && l && acc, "a tensor argument is null");
    SAR_CHECK_ARG(tq || a_l, "either tq or a_l must be given");
    SAR_CHECK_ARG(aligned16(Zq) && aligned16(acc) && aligned16(a_l), "Zq, acc and a_l must be 16-byte aligned");
    const HeadGroups hg = head_groups(dtype, H, D);
    for (int g = 0; g < hg.n; ++g) {
        const size_t f0 = (size_t)g * hg.Fg, h0 = (size_t)g * hg.Hg;
        FwdArgs a{};
        a.indptr = k.indptr;
        a.indices = reinterpret_cast<const uint32_t*>(k.indices);
        a.rows = reinterpret_cast<const uint32_t*>(k.rows);
        a.n_rows = k.n_rows;
        a.n_long = k.n_long;
        a.Z = shift(Zq, f0 * hg.fb);
        a.t = tq ? tq + h0 : nullptr;
        a.a_l = tq ? nullptr : a_l + f0;
        a.s = s + h0;
        a.m = m + h0;
        a.l = l + h0;
        a.acc = acc + f0;
        a.H = hg.Hg;
        a.D = D;
        a.F = hg.Fg;
        a.ldz = H * D;
        a.ldh = H;
        a.slope = slope;
        PtrTab none{};
        SAR_DISPATCH_ROW(dtype, hg.fast_fwd ? hg.full : hg.piece,
                         SAR_TRY((launch_fwd<T, false>(a, none, none, 0, sar::as_stream(stream)))));
    }
    return SAR_OK;
}

extern "C" int sar_gat_fwd_end(const float* m, const float* l, const float* acc, int act, void* out, float* L,
                               int dtype, int64_t n_dst, int H, int D, void* stream)
{
    SAR_TRY(check_shape(dtype, H, D));
    SAR_TRY(check_act(act));
    SAR_CHECK_ARG(n_dst >= 0, "n_dst is negative");
    if (n_dst == 0) return SAR_OK;
    SAR_CHECK_ARG(m && l && acc && out && L, "a tensor argument is null");
    SAR_CHECK_ARG(aligned16(acc) && aligned16(out), "acc and out must be 16-byte aligned");
    const int F = H * D;
    const HeadGroups hg = head_groups(dtype, H, D);
    hipStream_t st = sar::as_stream(stream);
    for (int g = 0; g < hg.n; ++g) {
        const size_t f0 = (size_t)g * hg.Fg, h0 = (size_t)g * hg.Hg;
        SAR_DISPATCH_ROW(dtype, hg.piece,
                         SAR_DISPATCH_G(T, hg.Fg, (k_fwd_end<T, kG><<<nodewise_grid(n_dst, kWave / kG), kGatherThreads, 0, st>>>(
                                                      m + h0, l + h0, acc + f0, static_cast<T*>(out) + f0, L + h0, n_dst,
                                                      hg.Hg, D, hg.Fg, F, H, act))));
        SAR_LAUNCH_CHECK();
    }
    return SAR_OK;
}

extern "C" int sar_gat_fwd_all(const sar_blocks_t* b, const void* const* Zq, const float* s,
                               const float* const* tq, const float* a_l, int dtype, int H, int D, float slope,
                               int act, void* out, float* L, void* stream)
{
    SAR_CHECK_ARG(b != nullptr, "handle is null");
    SAR_TRY(check_shape(dtype, H, D));
    SAR_TRY(check_act(act));
    if (!b->f_indptr) return sar::fail(SAR_ERR_STATE, "handle was built without SAR_BUILD_FUSED");
    if (b->n_dst == 0) return SAR_OK;
    SAR_CHECK_ARG(Zq && s && out && L, "a tensor argument is null");
    SAR_CHECK_ARG(tq || a_l, "either tq or a_l must be given");
    SAR_CHECK_ARG(aligned16(out) && aligned16(a_l), "out and a_l must be 16-byte aligned");
    for (int q = 0; q < b->P; ++q) {
        SAR_CHECK_ARG((Zq[q] && (!tq || tq[q])) || b->blk[q].nnz == 0, "Zq[%d] or tq[%d] is null", q, q);
        SAR_CHECK_ARG(aligned16(Zq[q]), "Zq[%d] must be 16-byte aligned", q);
    }
    hipStream_t st = sar::as_stream(stream);
    const HeadGroups hg = head_groups(dtype, H, D);
    for (int g = 0; g < hg.n; ++g) {
        const size_t f0 = (size_t)g * hg.Fg, h0 = (size_t)g * hg.Hg;
        PtrTab zt{}, tt{};
        for (int q = 0; q < b->P; ++q) {
            zt.p[q] = shift(Zq[q], f0 * hg.fb);
            tt.p[q] = (tq && tq[q]) ? tq[q] + h0 : nullptr;
        }
        FwdArgs a{};
        a.indptr = b->f_indptr;
        a.indices = b->f_indices;
        a.rows = reinterpret_cast<const uint32_t*>(b->f_rows);
        a.n_rows = b->n_dst;   // the list ends with the destinations that have no in-edge: out = 0, L = -inf
        a.n_long = b->n_f_long;
        a.s = s + h0;
        a.a_l = tq ? nullptr : a_l + f0;
        a.out = shift(out, f0 * hg.fb);
        a.L = L + h0;
        a.H = hg.Hg;
        a.D = D;
        a.F = hg.Fg;
        a.ldz = H * D;
        a.ldh = H;
        a.tag_shift = b->tag_shift;
        a.slope = slope;
        a.act = act;
        SAR_DISPATCH_ROW(dtype, hg.fast_fwd ? hg.full : hg.piece, SAR_TRY((launch_fwd<T, true>(a, zt, tt, b->P, st))));
    }
    return SAR_OK;
}

extern "C" int sar_gat_workspace_bytes(int64_t n_dst, int64_t n_src_max, int H, int D, size_t* bytes)
{
    SAR_CHECK_ARG(bytes != nullptr, "bytes is null");
    SAR_CHECK_ARG(n_dst >= 0 && n_src_max >= 0 && H > 0 && D > 0, "sizes must be non-negative, H and D positive");
    *bytes = workspace_bytes(256);
    return SAR_OK;
}

extern "C" int sar_gat_bwd_begin(const void* G, const void* out, const float* s, const float* L, int act,
                                 void* Gact, int dtype, float* rec, float* ds, int64_t n_dst, int H, int D,
                                 void* stream)
{
    SAR_TRY(check_shape(dtype, H, D));
    SAR_TRY(check_act(act));
    SAR_CHECK_ARG(n_dst >= 0, "n_dst is negative");
    if (n_dst == 0) return SAR_OK;
    SAR_CHECK_ARG(G && out && s && L && rec && ds, "a tensor argument is null");
    SAR_CHECK_ARG(aligned16(G) && aligned16(out) && aligned16(rec), "G, out and rec must be 16-byte aligned");
    SAR_CHECK_ARG(act == SAR_ACT_NONE || (Gact && aligned16(Gact)), "a non-linearity needs Gact (16-byte aligned)");
    const int F = H * D;
    const HeadGroups hg = head_groups(dtype, H, D);
    hipStream_t st = sar::as_stream(stream);
    for (int g = 0; g < hg.n; ++g) {
        const size_t f0 = (size_t)g * hg.Fg, h0 = (size_t)g * hg.Hg;
        const void* Gg = shift(G, f0 * hg.fb);
        const void* og = shift(out, f0 * hg.fb);
        float4* recg = reinterpret_cast<float4*>(rec) + h0;
        SAR_DISPATCH_ROW(dtype, hg.piece,
                         SAR_DISPATCH_G(T, hg.Fg, (k_bwd_begin<T, kG><<<nodewise_grid(n_dst, kWave / kG), kGatherThreads, 0, st>>>(
                                                      static_cast<const T*>(Gg), static_cast<const T*>(og), s + h0, L + h0,
                                                      recg, ds + h0, n_dst, hg.Hg, D, hg.Fg, F, H, act,
                                                      static_cast<T*>(shift(Gact, f0 * hg.fb))))));
        SAR_LAUNCH_CHECK();
    }
    return SAR_OK;
}

namespace {

int bwd_common_checks(const sar_blocks_t* b, int dtype, int H, int D, const void* G, const float* rec,
                      const float* a_l, const float* ds, const float* da_l, const void* work, size_t work_bytes)
{
    SAR_CHECK_ARG(b != nullptr, "handle is null");
    SAR_TRY(check_shape(dtype, H, D));
    if (!(b->flags & SAR_BUILD_TRANSPOSE))
        return sar::fail(SAR_ERR_STATE, "handle was built without SAR_BUILD_TRANSPOSE");
    // with no destination at all the destination-side tensors have no element (and may be null):
    // the sources still get their zero rows
    SAR_CHECK_ARG(a_l && da_l && (b->n_dst == 0 || (G && rec && ds)), "a tensor argument is null");
    SAR_CHECK_ARG(aligned16(G) && aligned16(rec) && aligned16(a_l), "G, rec and a_l must be 16-byte aligned");
    SAR_CHECK_ARG(work != nullptr && aligned16(work), "work is null or not 16-byte aligned");
    const size_t need = workspace_bytes(256);
    SAR_CHECK_ARG(work_bytes >= need, "work_bytes=%zu is below the %zu bytes required", work_bytes, need);
    return SAR_OK;
}

// Fields that do not depend on the block(s) or on the head group.
void fill_bwd_group(BwdScalars& a, const HeadGroups& hg, int g, int H, int D, const void* G, const float* rec,
                    const float* a_l, float* ds, void* work, float slope)
{
    const size_t f0 = (size_t)g * hg.Fg, h0 = (size_t)g * hg.Hg;
    a.G = shift(G, f0 * hg.fb);
    a.rec = reinterpret_cast<const float4*>(rec) + h0;
    a.a_l = a_l + f0;
    a.ds = ds + h0;
    a.partial = static_cast<float*>(work);
    a.H = hg.Hg;
    a.D = D;
    a.F = hg.Fg;
    a.ldz = H * D;
    a.ldh = H;
    a.slope = slope;
}

}  // namespace

extern "C" int sar_gat_bwd_block(const sar_blocks_t* b, int q, const void* Zq, const void* G, const float* tq,
                                 const float* rec, const float* a_l, int dtype, int H, int D, float slope,
                                 void* dZq, float* dtq, float* ds, float* da_l, void* work, size_t work_bytes,
                                 void* stream)
{
    SAR_TRY(bwd_common_checks(b, dtype, H, D, G, rec, a_l, ds, da_l, work, work_bytes));
    SAR_CHECK_ARG(q >= 0 && q < b->P, "block %d out of range [0,%d)", q, b->P);
    const sar::Block& k = b->blk[q];
    if (k.n_src == 0 || (sar::skips_untouched(b->flags) && k.n_t_rows == 0)) return SAR_OK;
    SAR_CHECK_ARG(Zq && dZq, "a tensor argument is null");
    SAR_CHECK_ARG(aligned16(Zq) && aligned16(dZq), "Zq and dZq must be 16-byte aligned");
    hipStream_t st = sar::as_stream(stream);
    const HeadGroups hg = head_groups(dtype, H, D);
    for (int g = 0; g < hg.n; ++g) {
        const size_t f0 = (size_t)g * hg.Fg, h0 = (size_t)g * hg.Hg;
        BwdArgs tabs{};
        tabs.t_indptr[0] = k.t_indptr;
        tabs.t_indices[0] = k.t_indices;
        tabs.Z[0] = shift(Zq, f0 * hg.fb);
        tabs.t[0] = tq ? tq + h0 : nullptr;
        tabs.dZ[0] = shift(dZq, f0 * hg.fb);
        tabs.dt[0] = dtq ? dtq + h0 : nullptr;
        tabs.rank[0] = (b->flags & SAR_BUILD_COMPACT) ? k.t_rank : nullptr;
        BwdScalars a{};
        a.rows = reinterpret_cast<const uint32_t*>(k.t_rows);
        // sources without edges come last and get dZ = 0, dt = 0, unless the handle skips them
        a.n_rows = sar::skips_untouched(b->flags) ? k.n_t_rows : k.n_src;
        a.n_long = k.n_t_long;
        a.n_wide = k.n_t_wide;
        a.n_touched = k.n_t_rows;
        a.n_src_host = &k.n_src;
        a.n_blocks = 1;
        fill_bwd_group(a, hg, g, H, D, G, rec, a_l, ds, work, slope);
        SAR_DISPATCH_ROW(dtype, hg.fast_bwd ? hg.full : hg.piece, SAR_TRY((launch_bwd<T, false>(tabs, a, da_l + f0, st))));
    }
    return SAR_OK;
}

extern "C" int sar_gat_bwd_all(const sar_blocks_t* b, const void* const* Zq, const void* G,
                               const float* const* tq, const float* rec, const float* a_l, int dtype, int H,
                               int D, float slope, void* const* dZq, float* const* dtq, float* ds, float* da_l,
                               void* work, size_t work_bytes, void* stream)
{
    SAR_TRY(bwd_common_checks(b, dtype, H, D, G, rec, a_l, ds, da_l, work, work_bytes));
    SAR_CHECK_ARG(Zq && dZq, "a pointer table is null");
    if (b->P > SAR_MAX_BLOCKS)
        return sar::fail(SAR_ERR_UNSUPPORTED, "an all-blocks call takes at most %d blocks, the handle has %d: use the "
                         "per-block calls", SAR_MAX_BLOCKS, b->P);
    hipStream_t st = sar::as_stream(stream);
    for (int q = 0; q < b->P; ++q) {
        if (b->blk[q].n_src == 0 || (sar::skips_untouched(b->flags) && b->blk[q].n_t_rows == 0)) continue;
        SAR_CHECK_ARG(Zq[q] && (!tq || tq[q]) && dZq[q] && (!dtq || dtq[q]), "a tensor of block %d is null", q);
        SAR_CHECK_ARG(aligned16(Zq[q]) && aligned16(dZq[q]), "Zq[%d] and dZq[%d] must be 16-byte aligned", q, q);
    }
    const HeadGroups hg = head_groups(dtype, H, D);
    int64_t n_src_all[SAR_MAX_BLOCKS];
    for (int q = 0; q < b->P; ++q) n_src_all[q] = b->blk[q].n_src;
    for (int g = 0; g < hg.n; ++g) {
        const size_t f0 = (size_t)g * hg.Fg, h0 = (size_t)g * hg.Hg;
        BwdArgs tabs{};
        for (int q = 0; q < b->P; ++q) {
            const sar::Block& k = b->blk[q];
            if (k.n_src == 0) continue;
            tabs.t_indptr[q] = k.t_indptr;
            tabs.t_indices[q] = k.t_indices;
            tabs.Z[q] = shift(Zq[q], f0 * hg.fb);
            tabs.t[q] = tq ? tq[q] + h0 : nullptr;
            tabs.dZ[q] = shift(dZq[q], f0 * hg.fb);
            tabs.dt[q] = dtq ? dtq[q] + h0 : nullptr;
            tabs.rank[q] = (b->flags & SAR_BUILD_COMPACT) ? k.t_rank : nullptr;
        }
        BwdScalars a{};
        a.rows = b->ft_rows;
        a.n_rows = 0;
        for (int q = 0; q < b->P; ++q) a.n_rows += b->blk[q].n_src;
        if (sar::skips_untouched(b->flags)) a.n_rows = b->n_ft_rows;
        a.n_wide = b->n_ft_wide;
        a.n_touched = b->n_ft_rows;
        a.n_single = b->n_single;
        a.s_dst = b->s_dst;
        a.s_src = b->s_src;
        a.s_row = b->s_row;
        a.n_src_host = n_src_all;
        a.n_blocks = b->P;
        a.n_long = b->n_ft_long;
        a.tag_shift = b->tag_shift;
        fill_bwd_group(a, hg, g, H, D, G, rec, a_l, ds, work, slope);
        SAR_DISPATCH_ROW(dtype, hg.fast_bwd ? hg.full : hg.piece, SAR_TRY((launch_bwd<T, true>(tabs, a, da_l + f0, st))));
    }
    return SAR_OK;
}

namespace {

// Scratch of the entry point that allocates nothing: one row of partial sums of da_r per
// workgroup of k_bwd_end (at most kMaxPersistentWGs workgroups, at most 512 values per launch).
// Host code never uses the array's name as an address: the device address is looked up once
// per device (scratch_of) and passed to the kernels like any caller workspace.
constexpr size_t kScratchFloats = (size_t)kMaxPersistentWGs * 512;
static __device__ __align__(256) float scratch[kScratchFloats];

constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (each device holds its own copy).
int scratch_of(float** out)
{
    int dev = -1;
    SAR_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return sar::fail(SAR_ERR_UNSUPPORTED, "device ordinal %d is beyond %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        SAR_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return sar::fail(SAR_ERR_HIP, "hipGetSymbolAddress returned a null address for the scratch array");
        g_scratch_ptr[dev] = static_cast<float*>(p);
    }
    *out = g_scratch_ptr[dev];
    return SAR_OK;
}

// partial: room for one row of hg.Fg sums per workgroup; partial_floats = its size in values.
int bwd_end_impl(const void* Zdst, const float* ds, const float* a_r, const void* dZadd,
                 const int32_t* dZadd_rank, void* dZdst, float* da_r, int dtype, int64_t n_dst, int H, int D, float* partial, size_t partial_floats,
                 hipStream_t st)
{
    const int F = H * D;
    const HeadGroups hg = head_groups(dtype, H, D);
    for (int g = 0; g < hg.n; ++g) {
        const size_t f0 = (size_t)g * hg.Fg, h0 = (size_t)g * hg.Hg;
        unsigned grid = 1;
        const int slots = kWave / lanes_for(hg.Fg, hg.piece);
        grid = nodewise_grid(n_dst, slots);
        if ((size_t)grid * hg.Fg > partial_floats)
            return sar::fail(SAR_ERR_UNSUPPORTED, "%u workgroups x %d partial sums exceed the %zu values of scratch",
                             grid, hg.Fg, partial_floats);
        SAR_DISPATCH_ROW(dtype, hg.piece,
                         SAR_DISPATCH_G(T, hg.Fg, (k_bwd_end<T, kG><<<grid, kGatherThreads, 0, st>>>(
                                                      static_cast<const T*>(Zdst) + f0, ds + h0, a_r + f0,
                                                      dZadd ? static_cast<const T*>(dZadd) + f0 : nullptr, dZadd_rank,
                                                      dZdst ? static_cast<T*>(dZdst) + f0 : nullptr, partial, n_dst,
                                                      hg.Hg, D, hg.Fg, F, H))));
        SAR_LAUNCH_CHECK();
        k_reduce_partials<<<hg.Fg, 256, 0, st>>>(partial, (int)grid, hg.Fg, da_r + f0);
        SAR_LAUNCH_CHECK();
    }
    return SAR_OK;
}

int bwd_end_checks(const void* Zdst, const float* ds, const float* a_r, const void* dZadd,
                   const int32_t* dZadd_rank, void* dZdst, float* da_r, int dtype, int64_t n_dst, int H, int D)
{
    SAR_CHECK_ARG(!dZadd_rank || (dZadd && dZadd != dZdst), "dZadd_rank needs a dZadd that is not dZdst");
    SAR_TRY(check_shape(dtype, H, D));
    SAR_CHECK_ARG(n_dst >= 0, "n_dst is negative");
    if (n_dst == 0) return SAR_OK;
    SAR_CHECK_ARG(Zdst && ds && a_r && da_r, "a tensor argument is null");
    SAR_CHECK_ARG(aligned16(Zdst) && aligned16(dZdst) && aligned16(dZadd),
                  "Zdst, dZadd and dZdst must be 16-byte aligned");
    return SAR_OK;
}

}  // namespace

extern "C" int sar_gat_bwd_end(const void* Zdst, const float* ds, const float* a_r, const void* dZadd,
                               const int32_t* dZadd_rank, void* dZdst, float* da_r, int dtype, int64_t n_dst,
                               int H, int D, void* work, size_t work_bytes, void* stream)
{
    SAR_TRY(bwd_end_checks(Zdst, ds, a_r, dZadd, dZadd_rank, dZdst, da_r, dtype, n_dst, H, D));
    if (n_dst == 0) return SAR_OK;
    SAR_CHECK_ARG(work != nullptr && aligned16(work), "work is null or not 16-byte aligned");
    const size_t need = workspace_bytes(256);
    SAR_CHECK_ARG(work_bytes >= need, "work_bytes=%zu is below the %zu bytes required", work_bytes, need);
    return bwd_end_impl(Zdst, ds, a_r, dZadd, dZadd_rank, dZdst, da_r, dtype, n_dst, H, D,
                        static_cast<float*>(work), work_bytes / sizeof(float), sar::as_stream(stream));
}

extern "C" int sar_gat_bwd_end_noalloc(const void* Zdst, const float* ds, const float* a_r, const void* dZadd,
                                       const int32_t* dZadd_rank, void* dZdst, float* da_r, int dtype,
                                       int64_t n_dst, int H, int D, void* stream)
{
    SAR_TRY(bwd_end_checks(Zdst, ds, a_r, dZadd, dZadd_rank, dZdst, da_r, dtype, n_dst, H, D));
    if (n_dst == 0) return SAR_OK;
    float* partial = nullptr;
    SAR_TRY(scratch_of(&partial));
    return bwd_end_impl(Zdst, ds, a_r, dZadd, dZadd_rank, dZdst, da_r, dtype, n_dst, H, D, partial,
                        kScratchFloats, sar::as_stream(stream));
}
