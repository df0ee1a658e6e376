// Fused attention kernels specialised for rows of F = 256 values (1 KiB fp32 or
// 512 B bf16): the whole wavefront covers one row, lane x owns features
// 4x..4x+3, and a head is a group of LPH = D/4 consecutive lanes.
//
// Per-edge scalars (score, softmax weight, score gradient) are not computed
// redundantly by every lane of a head.  Edges are taken in sub-batches of up
// to B, and inside a head group lane k works on edge k of the sub-batch: the
// scores of B edges x H heads are formed by one instruction stream, then each
// weight is broadcast back to its head group (DS_SWIZZLE) for the
// multiply-add with the gathered row.  Row addresses come from scalar
// registers (V_READLANE of the coalesced index chunk), so the gathers are
// SGPR-base + lane-offset loads with up to B rows in flight per wavefront.
//
// Two lane geometries.  Exact: the row is 256 contiguous values, lane x owns
// 4x..4x+3.  Padded (template flag PAD): the launch covers 64/LPH heads of any
// width D <= 4*LPH (D a multiple of 4) inside rows of stride `ld`; head h sits in
// lanes [h*LPH, (h+1)*LPH), lane k of it owns features h*D + 4k.. while 4k < D
// and is idle otherwise (it still takes its turn at the per-edge scalars).  That
// brings head widths such as 100 and rows wider than one wavefront (several
// launches over groups of heads) onto these kernels.
#pragma once

#include <type_traits>

#include "../../include/sar_mi355x.h"
#include "gather_common.h"
#include "sar_internal.h"

namespace sar {
namespace f256 {

constexpr int kF = 256;

// ---- cross-lane helpers (wave64, DPP rows of 16 lanes) --------------------

template <int CTRL>
__device__ inline float dpp(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ inline int dpp_i(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
constexpr int kRowShr = 0x110;         // + n: lane r of a row of 16 reads lane r - n (0 where there is none)
constexpr int kRowShl = 0x100;         // + n: lane r reads lane r + n
constexpr int kQuadXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kQuadXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kRowHalfMirror = 0x141;
constexpr int kRowRor4 = 0x124;
constexpr int kRowRor8 = 0x128;

template <int PATTERN>
__device__ inline float swizzle(float v)
{
    return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), PATTERN));
}

struct OpSum {
    static __device__ inline float f(float a, float b) { return a + b; }
};
struct OpMax {
    static __device__ inline float f(float a, float b) { return fmaxf(a, b); }
};

// All-reduce over each group of LPH consecutive lanes (LPH = 1..64, power of two).
template <int LPH, typename Op>
__device__ inline float group_all(float v)
{
    if constexpr (LPH >= 2) v = Op::f(v, dpp<kQuadXor1>(v));
    if constexpr (LPH >= 4) v = Op::f(v, dpp<kQuadXor2>(v));
    if constexpr (LPH == 8) v = Op::f(v, dpp<kRowHalfMirror>(v));
    if constexpr (LPH >= 16) {
        v = Op::f(v, dpp<kRowRor4>(v));
        v = Op::f(v, dpp<kRowRor8>(v));
    }
    if constexpr (LPH >= 32) v = Op::f(v, swizzle<0x401F>(v));   // xor 16
    if constexpr (LPH >= 64) v = Op::f(v, __shfl_xor(v, 32));
    return v;
}

// Value held by lane K of the caller's head group, delivered to the whole group.
template <int LPH, int K>
__device__ inline float group_bcast(float v)
{
    if constexpr (LPH >= 64) {
        return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), K));
    } else {
        constexpr int kAnd = (LPH >= 32) ? 0x00 : (0x1F & ~(LPH - 1));
        return swizzle<(K << 5) | kAnd>(v);
    }
}

// Sums of 8 per-lane values over each group of LPH consecutive lanes, one sum per lane: the lane
// at position k of its group (k % 8 for LPH > 8) returns the group's sum of c[k % 8].  Eight
// separate all-reductions would move every value through every step; here the lanes first split
// the eight values between them while they add (pairs, quads, eights: 4 + 2 + 1 exchanges), and
// only one value per lane takes the remaining log2(LPH / 8) steps.
// Measured: a gain from LPH = 32 on, where each all-reduction takes steps through the LDS crossbar
// (bf16 4 x 128 and 2 x 256: 3 to 10% per pass); within 16 lanes the eight independent DPP chains
// of the separate all-reductions are as fast or faster.
constexpr int kScatterSumsFrom = 32;
constexpr int kQuadReverse = 0x1B;     // quad_perm [3,2,1,0]
template <int LPH>
__device__ inline float group_sums8(const float (&c)[8])
{
    static_assert(LPH >= 8, "eight lanes share eight sums");
    const int k = threadIdx.x;           // groups start at multiples of 8: the low bits are the position
    const bool b0 = k & 1, b1 = k & 2, b2 = k & 4;
    float v1[4], v2[2];
#pragma unroll
    for (int m = 0; m < 4; ++m) {        // the partner (lane ^ 1) takes the values of the other parity
        const float mine = b0 ? c[2 * m + 1] : c[2 * m], send = b0 ? c[2 * m] : c[2 * m + 1];
        v1[m] = mine + dpp<kQuadXor1>(send);
    }
#pragma unroll
    for (int n = 0; n < 2; ++n) {        // lane ^ 2
        const float mine = b1 ? v1[2 * n + 1] : v1[2 * n], send = b1 ? v1[2 * n] : v1[2 * n + 1];
        v2[n] = mine + dpp<kQuadXor2>(send);
    }
    const float mine = b2 ? v2[1] : v2[0], send = b2 ? v2[0] : v2[1];
    // lane ^ 4 = the mirror image within 8 lanes (lane ^ 7) of the quad's reverse (lane ^ 3)
    float v = mine + dpp<kQuadReverse>(dpp<kRowHalfMirror>(send));
    if constexpr (LPH >= 16) v += dpp<kRowRor8>(v);
    if constexpr (LPH >= 32) v += swizzle<0x401F>(v);   // xor 16
    if constexpr (LPH >= 64) v += __shfl_xor(v, 32);
    return v;
}

template <int N, typename Fn>
__device__ inline void static_for(Fn&& fn)
{
    if constexpr (N > 0) {
        static_for<N - 1>(fn);
        fn(std::integral_constant<int, N - 1>{});
    }
}

// ---- row access: 4 values per lane ---------------------------------------

template <typename T>
struct Row4;
template <>
struct Row4<float> {
    using Raw = float4;
    static __device__ inline Raw load(const float* row, int lane) { return reinterpret_cast<const float4*>(row)[lane]; }
    static __device__ inline void unpack(const Raw& r, float (&v)[4])
    {
        v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
    }
    static __device__ inline void store(float* row, int lane, const float (&v)[4])
    {
        reinterpret_cast<float4*>(row)[lane] = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <>
struct Row4<bf16_t> {
    using Raw = uint2;
    static __device__ inline Raw load(const bf16_t* row, int lane) { return reinterpret_cast<const uint2*>(row)[lane]; }
    static __device__ inline void unpack(const Raw& r, float (&v)[4])
    {
        v[0] = __uint_as_float(r.x << 16);
        v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16);
        v[3] = __uint_as_float(r.y & 0xffff0000u);
    }
    static __device__ inline void store(bf16_t* row, int lane, const float (&v)[4])
    {
        uint2 r;
        r.x = pack2_bf16(v[0], v[1]);
        r.y = pack2_bf16(v[2], v[3]);
        reinterpret_cast<uint2*>(row)[lane] = r;
    }
};

// The lane's 4 values of a row (zeros for an idle lane of the padded geometry).
template <typename T, bool PAD>
__device__ inline typename Row4<T>::Raw load_lane(const T* row, int foff, bool on)
{
    using Raw = typename Row4<T>::Raw;
    if constexpr (PAD) {
        Raw r{};
        if (on) r = *reinterpret_cast<const Raw*>(row + foff);
        return r;
    } else {
        return *reinterpret_cast<const Raw*>(row + foff);
    }
}
template <typename T, bool PAD>
__device__ inline void store_lane(T* row, int foff, bool on, const float (&v)[4])
{
    if (!PAD || on) Row4<T>::store(row + foff, 0, v);
}

struct Tabs {
    const void* Z[SAR_MAX_BLOCKS];
    const float* t[SAR_MAX_BLOCKS];
};

__device__ inline float leaky2(float u, float slope) { return u > 0.f ? u : slope * u; }

// ------------------------------------------------------------------ forward

struct FwdP {
    const int32_t* indptr;
    const uint32_t* indices;
    const uint32_t* rows;
    int64_t n_rows, n_long;
    const void* Z;
    const float* t;      // source score halves, or null with FLY (formed from a_l and the gathered row)
    const float* a_l;
    const float* s;
    float* m;
    float* l;
    float* acc;
    void* out;
    float* L;
    int H;
    int tag_shift;
    float slope;
    int act;             // SAR_ACT_*: applied to the normalised output rows (ALL only)
    int ld, ldh, D;      // padded geometry: row stride (values), stride of the per-head arrays, head width
};

template <int LPH>
struct FwdState {
    float m2;       // running maximum (log2 units), uniform inside a head group
    float l;        // this lane's share of the running denominator
    float acc[4];   // running numerator for the lane's 4 features
};

// One 64-edge chunk position `mine`(lane) holds; folds edges [0,cnt) of it.
template <typename T, int LPH, int B, bool ALL, bool FLY, bool PAD>
__device__ inline void fwd_chunk(FwdState<LPH>& st, const FwdP& a, const Tabs& tabs, uint32_t mine, int cnt,
                                 int foff, bool on, int h, int k, float s2, const float (&al)[4])
{
    const int ld = PAD ? a.ld : kF, ldh = PAD ? a.ldh : a.H;
    const uint32_t mask = ALL ? ((1u << a.tag_shift) - 1u) : 0xffffffffu;
    for (int k0 = 0; k0 < cnt; k0 += B) {
        const int nb = min(B, cnt - k0);
        // gathers of the B source rows (a short last batch repeats its last edge; weight 0)
        typename Row4<T>::Raw raw[B];
        static_for<B>([&](auto kk) {
            const int e = k0 + min((int)decltype(kk)::value, nb - 1);
            const uint32_t id = (uint32_t)__builtin_amdgcn_readlane((int)mine, e);
            const T* zb = static_cast<const T*>(ALL ? tabs.Z[id >> a.tag_shift] : a.Z);
            raw[decltype(kk)::value] = load_lane<T, PAD>(zb + (int64_t)(id & mask) * ld, foff, on);
        });
        // scores: lane k of every head group takes edge k0+k
        const bool valid = k < nb;
        float tv = 0.f;
        if constexpr (FLY) {
            // t_j = <a_l, z_j> from the row just gathered; lane k keeps edge k's value
            float cs[B];
            static_for<B>([&](auto kk) {
                float v[4];
                Row4<T>::unpack(raw[decltype(kk)::value], v);
                float c = al[0] * v[0];
#pragma unroll
                for (int x = 1; x < 4; ++x) c = fmaf(al[x], v[x], c);
                cs[decltype(kk)::value] = c;
            });
            if constexpr (B == 8 && LPH >= kScatterSumsFrom) {
                tv = group_sums8<LPH>(cs);
            } else {
                static_for<B>([&](auto kk) {
                    const float c = group_all<LPH, OpSum>(cs[decltype(kk)::value]);
                    tv = (k == decltype(kk)::value) ? c : tv;
                });
            }
        } else {
            const uint32_t my = (uint32_t)__shfl((int)mine, k0 + (valid ? k : 0));
            const float* tb = ALL ? tabs.t[my >> a.tag_shift] : a.t;
            tv = tb[(int64_t)(my & mask) * ldh + h];
        }
        const float e2 = valid ? leaky2(fmaf(tv, kLog2e, s2), a.slope) : -INFINITY;
        const float cmax = group_all<LPH, OpMax>(e2);
        if (__builtin_amdgcn_ballot_w64(cmax > st.m2)) {
            const float mn = fmaxf(st.m2, cmax);
            const float c = fast_exp2(st.m2 - mn);    // first edges: exp2(-inf) = 0
            st.l *= c;
#pragma unroll
            for (int x = 0; x < 4; ++x) st.acc[x] *= c;
            st.m2 = mn;
        }
        const float p = fast_exp2(e2 - st.m2);        // 0 for the lanes without an edge
        st.l += p;
        static_for<B>([&](auto kk) {
            const float pk = group_bcast<LPH, decltype(kk)::value>(p);
            float v[4];
            Row4<T>::unpack(raw[decltype(kk)::value], v);
#pragma unroll
            for (int x = 0; x < 4; ++x) st.acc[x] = fmaf(pk, v[x], st.acc[x]);
        });
    }
}

template <typename T, int LPH, int B, bool ALL, bool FLY, bool PAD>
__global__ __launch_bounds__(kGatherThreads) void k_gat_fwd_f256(FwdP a, Tabs tabs)
{
    static_assert(B <= LPH, "a sub-batch must fit a head group");
    __shared__ float part[kWavesPerWG][kWave][6];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Padded geometry: a launch of fewer than 64/LPH heads leaves whole head groups without a head.
    // Such a group reads what the last head reads (valid memory), speaks for no edge and owns no
    // output: its lanes' `k` matches no slot, so every weight it forms is zero.
    const int h_pos = lane / LPH, k_pos = lane % LPH;
    const bool head_ok = !PAD || h_pos < a.H;
    const int h = head_ok ? h_pos : a.H - 1, k = head_ok ? k_pos : kWave;
    const int ld = PAD ? a.ld : kF, ldh = PAD ? a.ldh : a.H;
    const int foff = PAD ? h * a.D + 4 * k_pos : lane * 4;
    const bool on = PAD ? head_ok && 4 * k_pos < a.D : true;
    T* outp = static_cast<T*>(a.out);
    float al[4] = {0.f, 0.f, 0.f, 0.f};
    if constexpr (FLY) {
        if (on) load_f32<4>(a.a_l + foff, al);
    }

    auto init = [&](FwdState<LPH>& st, int i, bool carry) {
        st.m2 = -INFINITY;
        st.l = 0.f;
#pragma unroll
        for (int x = 0; x < 4; ++x) st.acc[x] = 0.f;
        if constexpr (!ALL) {
            if (carry) {   // state carried from the blocks already aggregated
                st.m2 = a.m[(int64_t)i * ldh + h] * kLog2e;
                st.l = (k == 0) ? a.l[(int64_t)i * ldh + h] : 0.f;
                if (on) load_f32<4>(a.acc + (int64_t)i * ld + foff, st.acc);
            }
        }
    };
    auto finish = [&](FwdState<LPH>& st, int i) {
        const float l = group_all<LPH, OpSum>(st.l);
        if constexpr (ALL) {
            const float inv = l > 0.f ? 1.f / l : 0.f;
            float v[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                v[x] = st.acc[x] * inv;
                if (a.act == SAR_ACT_RELU) v[x] = fmaxf(v[x], 0.f);
            }
            store_lane<T, PAD>(outp + (int64_t)i * ld, foff, on, v);
            if (k == 0) a.L[(int64_t)i * ldh + h] = l > 0.f ? (st.m2 + fast_log2(l)) * kLn2 : -INFINITY;
        } else {
            if (on) store_f32<4>(a.acc + (int64_t)i * ld + foff, st.acc);
            if (k == 0) {
                a.m[(int64_t)i * ldh + h] = st.m2 * kLn2;
                a.l[(int64_t)i * ldh + h] = l;
            }
        }
    };
    auto edges = [&](FwdState<LPH>& st, int i, int chunk0, int stride) {
        const float s2 = a.s[(int64_t)i * ldh + h] * kLog2e;
        const int beg = a.indptr[i], end = a.indptr[i + 1];
        for (int cb = beg + chunk0 * kWave; cb < end; cb += stride * kWave) {
            const int cnt = min(kWave, end - cb);
            const uint32_t mine = (lane < cnt) ? a.indices[cb + lane] : 0u;
            fwd_chunk<T, LPH, B, ALL, FLY, PAD>(st, a, tabs, mine, cnt, foff, on, h, k, s2, al);
        }
    };

    // the long rows at the head of the list: the four wavefronts share the row
    for (int64_t r = blockIdx.x; r < a.n_long; r += gridDim.x) {
        const int i = (int)a.rows[r];
        FwdState<LPH> st;
        init(st, i, wave == 0);
        edges(st, i, wave, kWavesPerWG);
        const float l = group_all<LPH, OpSum>(st.l);
#pragma unroll
        for (int x = 0; x < 4; ++x) part[wave][lane][x] = st.acc[x];
        part[wave][lane][4] = st.m2;
        part[wave][lane][5] = l;
        __syncthreads();
        if (wave == 0) {
            float m2 = st.m2, lt = l;
            for (int w = 1; w < kWavesPerWG; ++w) {
                const float om = part[w][lane][4], ol = part[w][lane][5];
                const float mn = fmaxf(m2, om);
                const float ref = (mn == -INFINITY) ? 0.f : mn;
                const float ca = fast_exp2(m2 - ref), cb = fast_exp2(om - ref);
                lt = lt * ca + ol * cb;
#pragma unroll
                for (int x = 0; x < 4; ++x) st.acc[x] = st.acc[x] * ca + part[w][lane][x] * cb;
                m2 = mn;
            }
            st.m2 = m2;
            st.l = (k == 0) ? lt : 0.f;
            finish(st, i);
        }
        __syncthreads();
    }
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerWG;
    for (int64_t r = a.n_long + (int64_t)blockIdx.x * kWavesPerWG + wave; r < a.n_rows; r += n_waves) {
        const int i = __builtin_amdgcn_readfirstlane((int)a.rows[r]);
        FwdState<LPH> st;
        init(st, i, true);
        edges(st, i, 0, 1);
        finish(st, i);
    }
}

// ----------------------------------------------------------------- backward

struct BwdTabs {
    const int32_t* t_indptr[SAR_MAX_BLOCKS];
    const int32_t* t_indices[SAR_MAX_BLOCKS];
    const void* Z[SAR_MAX_BLOCKS];
    const float* t[SAR_MAX_BLOCKS];
    void* dZ[SAR_MAX_BLOCKS];
    float* dt[SAR_MAX_BLOCKS];
    const int32_t* rank[SAR_MAX_BLOCKS];   // compact outputs: row of dZ / dt that source j owns (null: j itself)
};

struct BwdP {
    const uint32_t* rows;
    int64_t n_rows, n_long;
    const void* G;
    const float4* rec;
    const float* a_l;
    float* ds;
    float* partial;
    int H;
    int tag_shift;
    float slope;
    int ld, ldh, D;      // padded geometry, as in FwdP
};

struct BwdAcc4 {
    float dz[4];   // sum_i alpha G_i for the lane's 4 features
    float dt;      // this lane's share of sum_i du
};

template <typename T, int LPH, int B, bool PAD>
__device__ inline void bwd_chunk(BwdAcc4& ac, const BwdP& a, int mine, int cnt, int foff, bool on, int h, int k,
                                 const float (&zj)[4], float t2)
{
    const int ld = PAD ? a.ld : kF, ldh = PAD ? a.ldh : a.H;
    const T* Gp = static_cast<const T*>(a.G);
    for (int k0 = 0; k0 < cnt; k0 += B) {
        const int nb = min(B, cnt - k0);
        typename Row4<T>::Raw raw[B];
        static_for<B>([&](auto kk) {
            const int e = k0 + min((int)decltype(kk)::value, nb - 1);
            const int i = __builtin_amdgcn_readlane(mine, e);
            raw[decltype(kk)::value] = load_lane<T, PAD>(Gp + (int64_t)i * ld, foff, on);
        });
        const bool valid = k < nb;
        const int my_i = __shfl(mine, k0 + (valid ? k : 0));
        const float4 rec = a.rec[(int64_t)my_i * ldh + h];
        // c_k = <G_i, z_j> per head, reduced over the head's lanes; lane k keeps edge k's value
        float c_mine = 0.f;
        float cs[B];
        static_for<B>([&](auto kk) {
            float g[4];
            Row4<T>::unpack(raw[decltype(kk)::value], g);
            float c = g[0] * zj[0];
#pragma unroll
            for (int x = 1; x < 4; ++x) c = fmaf(g[x], zj[x], c);
            cs[decltype(kk)::value] = c;
        });
        if constexpr (B == 8 && LPH >= kScatterSumsFrom) {
            c_mine = group_sums8<LPH>(cs);
        } else {
            static_for<B>([&](auto kk) {
                const float c = group_all<LPH, OpSum>(cs[decltype(kk)::value]);
                c_mine = (k == decltype(kk)::value) ? c : c_mine;
            });
        }
        const float u2 = rec.x + t2;
        const float alpha = valid ? fast_exp2(leaky2(u2, a.slope) - rec.y) : 0.f;
        const float de = alpha * (c_mine - rec.z);
        const float du = u2 > 0.f ? de : a.slope * de;
        ac.dt += du;
        if (valid) unsafeAtomicAdd(a.ds + (int64_t)my_i * ldh + h, du);
        static_for<B>([&](auto kk) {
            const float ak = group_bcast<LPH, decltype(kk)::value>(alpha);
            float g[4];
            Row4<T>::unpack(raw[decltype(kk)::value], g);
#pragma unroll
            for (int x = 0; x < 4; ++x) ac.dz[x] = fmaf(ak, g[x], ac.dz[x]);
        });
    }
}

template <typename T, int LPH, int B, bool ALL, bool PAD>
__global__ __launch_bounds__(kGatherThreads) void k_gat_bwd_f256(BwdTabs tabs, BwdP a)
{
    static_assert(B <= LPH, "a sub-batch must fit a head group");
    __shared__ float part[kWavesPerWG][kWave][5];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Padded geometry: a launch of fewer than 64/LPH heads leaves whole head groups without a head.
    // Such a group reads what the last head reads (valid memory), speaks for no edge and owns no
    // output: its lanes' `k` matches no slot, so every weight it forms is zero.
    const int h_pos = lane / LPH, k_pos = lane % LPH;
    const bool head_ok = !PAD || h_pos < a.H;
    const int h = head_ok ? h_pos : a.H - 1, k = head_ok ? k_pos : kWave;
    const int ld = PAD ? a.ld : kF, ldh = PAD ? a.ldh : a.H;
    const int foff = PAD ? h * a.D + 4 * k_pos : lane * 4;
    const bool on = PAD ? head_ok && 4 * k_pos < a.D : true;
    const uint32_t mask = ALL ? ((1u << a.tag_shift) - 1u) : 0xffffffffu;

    float al[4] = {0.f, 0.f, 0.f, 0.f}, dal[4];
    if (on) load_f32<4>(a.a_l + foff, al);
#pragma unroll
    for (int x = 0; x < 4; ++x) dal[x] = 0.f;

    auto edges = [&](BwdAcc4& ac, int q, int j, int chunk0, int stride, float (&zj)[4]) {
        Row4<T>::unpack(load_lane<T, PAD>(static_cast<const T*>(tabs.Z[q]) + (int64_t)j * ld, foff, on), zj);
        float t2;
        if (tabs.t[q]) {
            t2 = tabs.t[q][(int64_t)j * ldh + h] * kLog2e;
        } else {   // t_j = <a_l, z_j> from the row this wavefront owns
            float c = al[0] * zj[0];
#pragma unroll
            for (int x = 1; x < 4; ++x) c = fmaf(al[x], zj[x], c);
            t2 = group_all<LPH, OpSum>(c) * kLog2e;
        }
        const int32_t* ip = tabs.t_indptr[q];
        const int32_t* idx = tabs.t_indices[q];
        const int beg = ip[j], end = ip[j + 1];
#pragma unroll
        for (int x = 0; x < 4; ++x) ac.dz[x] = 0.f;
        ac.dt = 0.f;
        for (int cb = beg + chunk0 * kWave; cb < end; cb += stride * kWave) {
            const int cnt = min(kWave, end - cb);
            const int mine = (lane < cnt) ? idx[cb + lane] : 0;
            bwd_chunk<T, LPH, B, PAD>(ac, a, mine, cnt, foff, on, h, k, zj, t2);
        }
    };
    // dZ_q[j] = sum alpha G + dt a_l ; dt_q[j] = dt ; da_l += dt z_j
    auto outputs = [&](const BwdAcc4& ac, float dt, int q, int j, const float (&zj)[4]) {
        float v[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            v[x] = fmaf(dt, al[x], ac.dz[x]);
            dal[x] = fmaf(dt, zj[x], dal[x]);
        }
        const int64_t jo = tabs.rank[q] ? tabs.rank[q][j] : j;
        store_lane<T, PAD>(static_cast<T*>(tabs.dZ[q]) + jo * ld, foff, on, v);
        if (k == 0 && tabs.dt[q]) tabs.dt[q][jo * ldh + h] = dt;
    };

    for (int64_t r = blockIdx.x; r < a.n_long; r += gridDim.x) {
        const uint32_t id = a.rows[r];
        const int q = ALL ? (int)(id >> a.tag_shift) : 0, j = (int)(id & mask);
        BwdAcc4 ac;
        float zj[4];
        edges(ac, q, j, wave, kWavesPerWG, zj);
        const float dt = group_all<LPH, OpSum>(ac.dt);
#pragma unroll
        for (int x = 0; x < 4; ++x) part[wave][lane][x] = ac.dz[x];
        part[wave][lane][4] = dt;
        __syncthreads();
        if (wave == 0) {
            float tot[5];
#pragma unroll
            for (int x = 0; x < 5; ++x) {
                float s = 0.f;
                for (int w = 0; w < kWavesPerWG; ++w) s += part[w][lane][x];
                tot[x] = s;
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) ac.dz[x] = tot[x];
            outputs(ac, tot[4], q, j, zj);
        }
        __syncthreads();
    }
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerWG;
    for (int64_t r = a.n_long + (int64_t)blockIdx.x * kWavesPerWG + wave; r < a.n_rows; r += n_waves) {
        const uint32_t id = (uint32_t)__builtin_amdgcn_readfirstlane((int)a.rows[r]);
        const int q = ALL ? (int)(id >> a.tag_shift) : 0, j = (int)(id & mask);
        BwdAcc4 ac;
        float zj[4];
        edges(ac, q, j, 0, 1, zj);
        outputs(ac, group_all<LPH, OpSum>(ac.dt), q, j, zj);
    }

    // this workgroup's share of da_l = sum_j dt_j z_j
    __syncthreads();
#pragma unroll
    for (int x = 0; x < 4; ++x) part[wave][lane][x] = dal[x];
    __syncthreads();
    if (wave == 0) {
        float v[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            float s = 0.f;
            for (int w = 0; w < kWavesPerWG; ++w) s += part[w][lane][x];
            v[x] = s;
        }
        store_f32<4>(a.partial + (int64_t)blockIdx.x * kF + lane * 4, v);
    }
}

// ------------------------------------------- backward, rows of few edges
//
// A source of fewer than 8 edges would leave most of a wide-kernel batch empty.  This kernel
// keeps the lane geometry of the wide kernel -- lane x owns
// features 4x..4x+3 of every row, so each row -- a source's own row, a gathered G row, the error
// row written back -- is one fully coalesced wave-wide access.  Independent work comes from
// taking S sources per wavefront at once: a round gathers B = S*R rows, R edges of each of the
// S sources, and lane k of every head group speaks for gather slot k (the edge's record,
// coefficient and score gradient), exactly as it speaks for edge k of a sub-batch in the wide
// kernel; slot k always belongs to source k / R, so a lane's share of dt needs no indexing.
//
// What describes a source is read ahead by the lanes themselves, one register per field:
// lane u*kAhead + e holds source u's list entry, edge range and output row, and the
// destination of its edge e.  List entries are read three groups ahead, ranges two, and
// destinations one, so that a group starts with its row gathers and no dependent chain.
template <typename T, int LPH, bool ALL, bool PAD>
__global__ __launch_bounds__(kGatherThreads) void k_gat_bwd_few(BwdTabs tabs, BwdP a, int64_t r_begin, int64_t r_end,
                                                                int partial_row0)
{
    constexpr int B = LPH >= 8 ? 8 : 4;   // gather slots per round
    constexpr int R = 2;                  // slots per source
    constexpr int S = B / R;              // sources per wavefront and group
    constexpr int kAhead = 8;             // edges per source whose destinations are read ahead: all of them
    static_assert(S * kAhead <= kWave, "one lane per (source, edge read ahead)");
    static_assert((1 << kNarrowMaxClass) <= kAhead, "this kernel's sources have fewer than kAhead edges");
    __shared__ float part[kWavesPerWG][kWave][4];
    __shared__ const void* s_Z[SAR_MAX_BLOCKS];
    __shared__ const float* s_t[SAR_MAX_BLOCKS];
    __shared__ void* s_dZ[SAR_MAX_BLOCKS];
    __shared__ float* s_dt[SAR_MAX_BLOCKS];
    __shared__ const int32_t* s_ip[SAR_MAX_BLOCKS];
    __shared__ const int32_t* s_ix[SAR_MAX_BLOCKS];
    __shared__ const int32_t* s_rank[SAR_MAX_BLOCKS];
    if (threadIdx.x < SAR_MAX_BLOCKS) {
        s_Z[threadIdx.x] = tabs.Z[threadIdx.x];
        s_t[threadIdx.x] = tabs.t[threadIdx.x];
        s_dZ[threadIdx.x] = tabs.dZ[threadIdx.x];
        s_dt[threadIdx.x] = tabs.dt[threadIdx.x];
        s_ip[threadIdx.x] = tabs.t_indptr[threadIdx.x];
        s_ix[threadIdx.x] = tabs.t_indices[threadIdx.x];
        s_rank[threadIdx.x] = tabs.rank[threadIdx.x];
    }
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // exact geometry: rows of 256 values; padded: heads of any width D <= 4 LPH inside rows of stride
    // ld, head groups beyond the launch's heads idle (see k_gat_fwd_f256)
    const int h_pos = lane / LPH, k_pos = lane % LPH;
    const bool head_ok = !PAD || h_pos < a.H;
    const int h = head_ok ? h_pos : a.H - 1, k = head_ok ? k_pos : kWave;
    const int ld = PAD ? a.ld : kF, ldh = PAD ? a.ldh : a.H;
    const int foff = PAD ? h * a.D + 4 * k_pos : lane * 4;
    const bool on = PAD ? head_ok && 4 * k_pos < a.D : true;
    const uint32_t mask = ALL ? ((1u << a.tag_shift) - 1u) : 0xffffffffu;
    const T* Gp = static_cast<const T*>(a.G);

    float al[4] = {0.f, 0.f, 0.f, 0.f}, dal[4];
    if (on) load_f32<4>(a.a_l + foff, al);
#pragma unroll
    for (int x = 0; x < 4; ++x) dal[x] = 0.f;

    // ---- the lanes' read-ahead of list entries, ranges and destinations
    const bool meta_lane = lane < S * kAhead;
    const int mu = lane / kAhead, me = lane % kAhead;
    const int64_t stride = (int64_t)gridDim.x * kWavesPerWG * S;
    struct Range { int q, j, beg, end, jo; };
    auto valid = [&](int64_t g) { return meta_lane && g + mu < r_end; };
    auto load_id = [&](int64_t g) -> uint32_t { return valid(g) ? a.rows[g + mu] : 0u; };
    auto load_range = [&](uint32_t id, int64_t g) {
        Range m{0, 0, 0, 0, 0};
        if (valid(g)) {
            m.q = ALL ? (int)(id >> a.tag_shift) : 0;
            m.j = (int)(id & mask);
            const int32_t* ip = s_ip[m.q];
            m.beg = ip[m.j];
            m.end = ip[m.j + 1];
            m.jo = s_rank[m.q] ? s_rank[m.q][m.j] : m.j;
        }
        return m;
    };
    auto load_dst = [&](const Range& m, int64_t g) { return (valid(g) && me < m.end - m.beg) ? s_ix[m.q][m.beg + me] : 0; };

    int64_t g0 = r_begin + ((int64_t)blockIdx.x * kWavesPerWG + wave) * S;
    uint32_t id2 = load_id(g0 + 2 * stride);
    Range m0 = load_range(load_id(g0), g0), m1 = load_range(load_id(g0 + stride), g0 + stride);
    int dst0 = load_dst(m0, g0);

    for (; g0 < r_end; g0 += stride) {
        const int dst1 = load_dst(m1, g0 + stride);
        const Range m2 = load_range(id2, g0 + 2 * stride);
        const uint32_t id3 = load_id(g0 + 3 * stride);

        // ---- the S sources of this group: uniform values out of the lanes that hold them
        bool have[S];
        int q[S], j[S], beg[S], end[S], jo[S];
        typename Row4<T>::Raw zr[S];
        int rounds = 0;
        static_for<S>([&](auto uu) {
            constexpr int u = decltype(uu)::value;
            have[u] = g0 + u < r_end;
            q[u] = __builtin_amdgcn_readlane(m0.q, u * kAhead);
            j[u] = __builtin_amdgcn_readlane(m0.j, u * kAhead);
            beg[u] = __builtin_amdgcn_readlane(m0.beg, u * kAhead);
            end[u] = __builtin_amdgcn_readlane(m0.end, u * kAhead);
            jo[u] = __builtin_amdgcn_readlane(m0.jo, u * kAhead);
            rounds = max(rounds, end[u] - beg[u]);
            zr[u] = typename Row4<T>::Raw{};
            if (have[u]) zr[u] = load_lane<T, PAD>(static_cast<const T*>(s_Z[q[u]]) + (int64_t)j[u] * ld, foff, on);
        });
        float t2[S], dz[S][4];
        static_for<S>([&](auto uu) {
            constexpr int u = decltype(uu)::value;
#pragma unroll
            for (int x = 0; x < 4; ++x) dz[u][x] = 0.f;
            t2[u] = 0.f;
            if (have[u]) {
                if (s_t[q[u]]) {
                    t2[u] = s_t[q[u]][(int64_t)j[u] * ldh + h] * kLog2e;
                } else {   // t_j = <a_l, z_j> from the row this wavefront holds
                    float zj[4];
                    Row4<T>::unpack(zr[u], zj);
                    float c = al[0] * zj[0];
#pragma unroll
                    for (int x = 1; x < 4; ++x) c = fmaf(al[x], zj[x], c);
                    t2[u] = group_all<LPH, OpSum>(c) * kLog2e;
                }
            }
        });
        // the source this lane's slot belongs to
        float t2_mine = t2[0];
        static_for<S>([&](auto uu) { t2_mine = (k / R == decltype(uu)::value) ? t2[decltype(uu)::value] : t2_mine; });
        float dt_mine = 0.f;

        for (int e = 0; e < rounds; e += R) {
            int dst[B];
            bool ok[B];
            typename Row4<T>::Raw raw[B];
            static_for<B>([&](auto kk) {
                constexpr int K = decltype(kk)::value, u = K / R, r = K % R;
                ok[K] = beg[u] + e + r < end[u];
                dst[K] = 0;
                raw[K] = typename Row4<T>::Raw{};
                if (ok[K]) dst[K] = __builtin_amdgcn_readlane(dst0, u * kAhead + e + r);
            });
            static_for<B>([&](auto kk) {
                constexpr int K = decltype(kk)::value;
                if (ok[K]) raw[K] = load_lane<T, PAD>(Gp + (int64_t)dst[K] * ld, foff, on);
            });
            // lane k speaks for slot k
            int my_i = 0;
            bool my_ok = false;
            static_for<B>([&](auto kk) {
                constexpr int K = decltype(kk)::value;
                my_i = (k == K) ? dst[K] : my_i;
                my_ok = (k == K) ? ok[K] : my_ok;
            });
            float4 rec = make_float4(0.f, INFINITY, 0.f, 0.f);   // L = +inf gives alpha = 0
            if (my_ok) rec = a.rec[(int64_t)my_i * ldh + h];
            float c_mine = 0.f;
            float cs[B];
            static_for<B>([&](auto kk) {
                constexpr int K = decltype(kk)::value;
                float g[4], zj[4];
                Row4<T>::unpack(raw[K], g);
                Row4<T>::unpack(zr[K / R], zj);
                float c = g[0] * zj[0];
#pragma unroll
                for (int x = 1; x < 4; ++x) c = fmaf(g[x], zj[x], c);
                cs[K] = c;
            });
            if constexpr (B == 8 && LPH >= kScatterSumsFrom) {
                c_mine = group_sums8<LPH>(cs);
            } else {
                static_for<B>([&](auto kk) {
                    constexpr int K = decltype(kk)::value;
                    const float c = group_all<LPH, OpSum>(cs[K]);
                    c_mine = (k == K) ? c : c_mine;
                });
            }
            const float u2 = rec.x + t2_mine;
            const float alpha = my_ok ? fast_exp2(leaky2(u2, a.slope) - rec.y) : 0.f;
            const float de = alpha * (c_mine - rec.z);
            const float du = u2 > 0.f ? de : a.slope * de;
            dt_mine += du;
            if (my_ok) unsafeAtomicAdd(a.ds + (int64_t)my_i * ldh + h, du);
            static_for<B>([&](auto kk) {
                constexpr int K = decltype(kk)::value;
                const float ak = group_bcast<LPH, K>(alpha);
                float g[4];
                Row4<T>::unpack(raw[K], g);
#pragma unroll
                for (int x = 0; x < 4; ++x) dz[K / R][x] = fmaf(ak, g[x], dz[K / R][x]);
            });
        }

        // ---- dZ_q[j] = sum alpha G + dt a_l ; dt_q[j] = dt ; da_l += dt z_j
        static_for<S>([&](auto uu) {
            constexpr int u = decltype(uu)::value;
            float dt = 0.f;
            static_for<R>([&](auto rr) { dt += group_bcast<LPH, u * R + decltype(rr)::value>(dt_mine); });
            if (have[u]) {
                float v[4], zj[4];
                Row4<T>::unpack(zr[u], zj);
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    v[x] = fmaf(dt, al[x], dz[u][x]);
                    dal[x] = fmaf(dt, zj[x], dal[x]);
                }
                store_lane<T, PAD>(static_cast<T*>(s_dZ[q[u]]) + (int64_t)jo[u] * ld, foff, on, v);
                if (k == 0 && s_dt[q[u]]) s_dt[q[u]][(int64_t)jo[u] * ldh + h] = dt;
            }
        });
        m0 = m1;
        dst0 = dst1;
        m1 = m2;
        id2 = id3;
    }

    // this workgroup's share of da_l
#pragma unroll
    for (int x = 0; x < 4; ++x) part[wave][lane][x] = dal[x];
    __syncthreads();
    if (wave == 0) {
        float v[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            float s = 0.f;
            for (int w = 0; w < kWavesPerWG; ++w) s += part[w][lane][x];
            v[x] = s;
        }
        store_f32<4>(a.partial + ((int64_t)partial_row0 + blockIdx.x) * kF + lane * 4, v);
    }
}

// ------------------------------------------- backward, sources of one edge
//
// A source with ONE edge in its block gains nothing from being walked source-major: its own row,
// its error row, and a gathered row of G with that destination's record, for one edge.  This
// kernel takes such edges in the order of their DESTINATIONS (a list the builder derives from the
// all-blocks index): the entries of a destination follow each other, so its row of G and its
// record come from the caches after the first of them, and what is left per edge is the source's
// row and one write of its error row -- which nobody else writes, so dZ_q[j] = alpha G_i + du a_l
// and dt_q[j] = du are plain stores.  Lane geometry and the sub-batch of B gather slots are those
// of the wide kernel; slot k here is an (edge, source) of its own and lane k of every head group
// speaks for it.
struct SingleP {
    const int32_t* dst;    // [n] destination of the entry's edge
    const uint32_t* src;   // [n] its source, tagged with the block
    const int32_t* row;    // [n] row of the source in its block's dZ_q / dt_q
    int64_t n;
};

template <typename T, int LPH, bool PAD>
__global__ __launch_bounds__(kGatherThreads) void k_gat_bwd_single(BwdTabs tabs, BwdP a, SingleP s, int partial_row0)
{
    constexpr int B = LPH >= 8 ? 8 : 4;
    static_assert(B <= LPH, "a sub-batch must fit a head group");
    __shared__ float part[kWavesPerWG][kWave][4];
    __shared__ const void* s_Z[SAR_MAX_BLOCKS];
    __shared__ const float* s_t[SAR_MAX_BLOCKS];
    __shared__ void* s_dZ[SAR_MAX_BLOCKS];
    __shared__ float* s_dt[SAR_MAX_BLOCKS];
    if (threadIdx.x < SAR_MAX_BLOCKS) {
        s_Z[threadIdx.x] = tabs.Z[threadIdx.x];
        s_t[threadIdx.x] = tabs.t[threadIdx.x];
        s_dZ[threadIdx.x] = tabs.dZ[threadIdx.x];
        s_dt[threadIdx.x] = tabs.dt[threadIdx.x];
    }
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // exact geometry: rows of 256 values; padded: heads of any width D <= 4 LPH inside rows of stride
    // ld, head groups beyond the launch's heads idle (see k_gat_fwd_f256)
    const int h_pos = lane / LPH, k_pos = lane % LPH;
    const bool head_ok = !PAD || h_pos < a.H;
    const int h = head_ok ? h_pos : a.H - 1, k = head_ok ? k_pos : kWave;
    const int ld = PAD ? a.ld : kF, ldh = PAD ? a.ldh : a.H;
    const int foff = PAD ? h * a.D + 4 * k_pos : lane * 4;
    const bool on = PAD ? head_ok && 4 * k_pos < a.D : true;
    const uint32_t mask = (1u << a.tag_shift) - 1u;
    const T* Gp = static_cast<const T*>(a.G);

    float al[4] = {0.f, 0.f, 0.f, 0.f}, dal[4];
    if (on) load_f32<4>(a.a_l + foff, al);
#pragma unroll
    for (int x = 0; x < 4; ++x) dal[x] = 0.f;

    // a wavefront takes 64 entries at a time, one per lane; the next 64 travel meanwhile
    const int64_t n_chunks = (s.n + kWave - 1) / kWave;
    const int64_t stride = (int64_t)gridDim.x * kWavesPerWG;
    struct Entry { int i; uint32_t id; int row; };
    auto load_entries = [&](int64_t c) {
        Entry e{0, 0u, 0};
        const int64_t at = c * kWave + lane;
        if (c < n_chunks && at < s.n) e = Entry{s.dst[at], s.src[at], s.row[at]};
        return e;
    };
    int64_t c = (int64_t)blockIdx.x * kWavesPerWG + wave;
    Entry cur = load_entries(c);
    for (; c < n_chunks; c += stride) {
        const Entry nxt = load_entries(c + stride);
        const int cnt = (int)min((int64_t)kWave, s.n - c * kWave);
        for (int k0 = 0; k0 < cnt; k0 += B) {
            const int nb = min(B, cnt - k0);
            int q[B], row[B];
            typename Row4<T>::Raw rg[B], rz[B];
            static_for<B>([&](auto kk) {
                constexpr int K = decltype(kk)::value;
                const int e = k0 + min(K, nb - 1);
                const int i = __builtin_amdgcn_readlane(cur.i, e);
                const uint32_t id = (uint32_t)__builtin_amdgcn_readlane((int)cur.id, e);
                q[K] = (int)(id >> a.tag_shift);
                row[K] = __builtin_amdgcn_readlane(cur.row, e);
                rg[K] = load_lane<T, PAD>(Gp + (int64_t)i * ld, foff, on);
                rz[K] = load_lane<T, PAD>(static_cast<const T*>(s_Z[q[K]]) + (int64_t)(id & mask) * ld, foff, on);
            });
            // lane k speaks for slot k
            const bool valid = k < nb;
            const int sel = k0 + (valid ? k : 0);
            const int my_i = __shfl(cur.i, sel);
            const uint32_t my_id = (uint32_t)__shfl((int)cur.id, sel);
            const int my_row = __shfl(cur.row, sel);
            const int my_q = (int)(my_id >> a.tag_shift);
            const float4 rec = a.rec[(int64_t)my_i * ldh + h];
            float cs[B], ts[B];
            static_for<B>([&](auto kk) {
                constexpr int K = decltype(kk)::value;
                float g[4], z[4];
                Row4<T>::unpack(rg[K], g);
                Row4<T>::unpack(rz[K], z);
                float cg = g[0] * z[0], ct = al[0] * z[0];
#pragma unroll
                for (int x = 1; x < 4; ++x) {
                    cg = fmaf(g[x], z[x], cg);
                    ct = fmaf(al[x], z[x], ct);
                }
                cs[K] = cg;
                ts[K] = ct;
            });
            float c_mine = 0.f, t_mine = 0.f;
            if constexpr (B == 8 && LPH >= kScatterSumsFrom) {
                c_mine = group_sums8<LPH>(cs);
                t_mine = group_sums8<LPH>(ts);
            } else {
                static_for<B>([&](auto kk) {
                    constexpr int K = decltype(kk)::value;
                    const float cg = group_all<LPH, OpSum>(cs[K]);
                    const float ct = group_all<LPH, OpSum>(ts[K]);
                    c_mine = (k == K) ? cg : c_mine;
                    t_mine = (k == K) ? ct : t_mine;
                });
            }
            if (valid && s_t[my_q]) t_mine = s_t[my_q][(int64_t)(my_id & mask) * ldh + h];
            const float u2 = rec.x + t_mine * kLog2e;
            const float alpha = valid ? fast_exp2(leaky2(u2, a.slope) - rec.y) : 0.f;
            const float de = alpha * (c_mine - rec.z);
            const float du = u2 > 0.f ? de : a.slope * de;
            if (valid && s_dt[my_q]) s_dt[my_q][(int64_t)my_row * ldh + h] = du;
            // ds_i += du: the entries of a destination follow each other, and a frequent destination
            // fills whole sub-batches: one atomic per run of slots that share the destination
            // (a running sum along the run, added by its last slot), not one per slot on one address
            {
                const int seg = valid ? my_i : -1 - k;
                float run = du;
                static_for<3>([&](auto ss) {
                    constexpr int sh = 1 << decltype(ss)::value;
                    if constexpr (sh < B) {
                        const float r_s = dpp<kRowShr + sh>(run);
                        const int i_s = dpp_i<kRowShr + sh>(seg);
                        if (k >= sh && i_s == seg) run += r_s;
                    }
                });
                const int next = dpp_i<kRowShl + 1>(seg);
                if (valid && (k == B - 1 || next != seg)) unsafeAtomicAdd(a.ds + (int64_t)my_i * ldh + h, run);
            }
            static_for<B>([&](auto kk) {
                constexpr int K = decltype(kk)::value;
                const float ak = group_bcast<LPH, K>(alpha);
                const float dk = group_bcast<LPH, K>(du);
                float g[4], z[4], v[4];
                Row4<T>::unpack(rg[K], g);
                Row4<T>::unpack(rz[K], z);
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    v[x] = fmaf(dk, al[x], ak * g[x]);
                    dal[x] = fmaf(dk, z[x], dal[x]);
                }
                if (K < nb) store_lane<T, PAD>(static_cast<T*>(s_dZ[q[K]]) + (int64_t)row[K] * ld, foff, on, v);
            });
        }
        cur = nxt;
    }

    // this workgroup's share of da_l
#pragma unroll
    for (int x = 0; x < 4; ++x) part[wave][lane][x] = dal[x];
    __syncthreads();
    if (wave == 0) {
        float v[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            float sum = 0.f;
            for (int w = 0; w < kWavesPerWG; ++w) sum += part[w][lane][x];
            v[x] = sum;
        }
        store_f32<4>(a.partial + ((int64_t)partial_row0 + blockIdx.x) * kF + lane * 4, v);
    }
}

}  // namespace f256
}  // namespace sar
