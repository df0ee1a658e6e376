// Partition-block builder: worker p's P destination-major CSR blocks
// G_{p,q} (Sec. 3.2 of the paper), plus the derived indexes the aggregation
// kernels launch from: the source-major transpose of every block, degree-class
// ordered row lists, the sorted touched-source list and the all-blocks row
// index.  Integer work only.  Every array whose content is part of the
// contract (indptr, indices, t_indptr, t_indices, deg, touched) is bit-exact
// and independent of scheduling: rows are filled through atomic cursors and
// then sorted.  Only the order inside a degree class of the launch lists is
// left to the scheduler.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "sar_internal.h"

namespace sar {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace sar

extern "C" const char* sar_last_error(void) { return sar::g_err; }
extern "C" int sar_version(void) { return 5; }

namespace {

using sar::Block;

constexpr int kThreads = 256;
constexpr int kScanTile = 2048;   // 256 threads x 8 values
constexpr int kPartTile = 1024;   // nodes per workgroup when ranking nodes in partitions
constexpr int kShortSort = 32;    // rows up to this length are insertion-sorted by one thread
constexpr int kLdsSort = 8192;    // longer rows up to this length are sorted in LDS

// ---------------------------------------------------------------- scan

__device__ inline int block_exclusive_scan(int v, int* lds4, int* total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    if (lane == 63) lds4[w] = incl;
    __syncthreads();
    int woff = 0;
    for (int k = 0; k < w; ++k) woff += lds4[k];
    *total = lds4[0] + lds4[1] + lds4[2] + lds4[3];
    __syncthreads();
    return woff + incl - v;
}

__global__ __launch_bounds__(kThreads) void k_tile_reduce(const int32_t* __restrict__ in, int64_t n,
                                                          int32_t* __restrict__ tile_sums)
{
    __shared__ int lds4[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + threadIdx.x * 8;
    int s = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k)
        if (base + k < n) s += in[base + k];
    int total;
    block_exclusive_scan(s, lds4, &total);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kThreads) void k_tile_scan(const int32_t* in, int64_t n,
                                                        const int32_t* __restrict__ tile_offsets,
                                                        int32_t* out)
{
    __shared__ int lds4[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + threadIdx.x * 8;
    int v[8], s = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        v[k] = (base + k < n) ? in[base + k] : 0;
        s += v[k];
    }
    int total;
    int run = block_exclusive_scan(s, lds4, &total) + (tile_offsets ? tile_offsets[blockIdx.x] : 0);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
    }
}

struct DeviceTemps {
    std::vector<void*> ptrs;
    ~DeviceTemps()
    {
        for (void* p : ptrs) (void)hipFree(p);
    }
    template <typename T>
    int alloc(T** out, int64_t count)
    {
        void* p = nullptr;
        SAR_HIP(hipMalloc(&p, std::max<int64_t>(count, 1) * sizeof(T)));
        ptrs.push_back(p);
        *out = static_cast<T*>(p);
        return SAR_OK;
    }
};

// out[k] = sum of in[0..k) for k in [0,n); in may equal out.
int exclusive_scan(const int32_t* in, int32_t* out, int64_t n, hipStream_t st, DeviceTemps& tmp)
{
    if (n <= 0) return SAR_OK;
    const int64_t tiles = (n + kScanTile - 1) / kScanTile;
    if (tiles == 1) {
        k_tile_scan<<<1, kThreads, 0, st>>>(in, n, nullptr, out);
        SAR_LAUNCH_CHECK();
        return SAR_OK;
    }
    int32_t* sums = nullptr;
    SAR_TRY(tmp.alloc(&sums, tiles));
    k_tile_reduce<<<(unsigned)tiles, kThreads, 0, st>>>(in, n, sums);
    SAR_LAUNCH_CHECK();
    SAR_TRY(exclusive_scan(sums, sums, tiles, st, tmp));
    k_tile_scan<<<(unsigned)tiles, kThreads, 0, st>>>(in, n, sums, out);
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

// ------------------------------------------------- local ids of all nodes

__global__ __launch_bounds__(kThreads) void k_part_tile_count(const int32_t* __restrict__ part,
                                                              int64_t N, int P, int64_t n_tiles,
                                                              int32_t* __restrict__ tile_counts,
                                                              int* __restrict__ err)
{
    static_assert(SAR_MAX_PARTS <= kThreads, "one thread per partition");
    __shared__ int hist[SAR_MAX_PARTS];
    if (threadIdx.x < SAR_MAX_PARTS) hist[threadIdx.x] = 0;
    __syncthreads();
    for (int r = 0; r < kPartTile / kThreads; ++r) {
        const int64_t v = (int64_t)blockIdx.x * kPartTile + r * kThreads + threadIdx.x;
        if (v < N) {
            const int pv = part[v];
            if (pv < 0 || pv >= P)
                atomicOr(err, 1);
            else
                atomicAdd(&hist[pv], 1);
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < P) tile_counts[(int64_t)threadIdx.x * n_tiles + blockIdx.x] = hist[threadIdx.x];
}

// lid[v] = number of nodes u < v in the same partition as v.
__global__ __launch_bounds__(kThreads) void k_local_ids(const int32_t* __restrict__ part, int64_t N,
                                                        int P, int64_t n_tiles,
                                                        const int32_t* __restrict__ tile_base,
                                                        int32_t* __restrict__ lid)
{
    constexpr int kRounds = kPartTile / kThreads;
    constexpr int kChunks = kPartTile / 64;
    __shared__ int cnt[kChunks][SAR_MAX_PARTS];
    for (int k = threadIdx.x; k < kChunks * SAR_MAX_PARTS; k += kThreads) (&cnt[0][0])[k] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int pv[kRounds], rank[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t v = (int64_t)blockIdx.x * kPartTile + r * kThreads + threadIdx.x;
        int x = (v < N) ? part[v] : -1;
        if (x < 0 || x >= P) x = -1;
        pv[r] = x;
        // lanes holding the same partition id find each other
        unsigned long long mine = 0;
        bool pending = x >= 0;
        unsigned long long todo = __ballot(pending);
        while (todo) {
            const int first = __ffsll((long long)todo) - 1;
            const int val = __shfl(x, first);
            const unsigned long long same = __ballot(pending && x == val);
            if (pending && x == val) {
                mine = same;
                pending = false;
            }
            todo = __ballot(pending);
        }
        const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        rank[r] = __popcll(mine & below);
        if (x >= 0 && rank[r] == 0) cnt[r * (kThreads / 64) + wave][x] = __popcll(mine);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t v = (int64_t)blockIdx.x * kPartTile + r * kThreads + threadIdx.x;
        if (pv[r] < 0) continue;
        const int chunk = r * (kThreads / 64) + wave;
        int pre = 0;
        for (int c = 0; c < chunk; ++c) pre += cnt[c][pv[r]];
        const int64_t col = (int64_t)pv[r] * n_tiles;
        lid[v] = tile_base[col + blockIdx.x] - tile_base[col] + pre + rank[r];
    }
}

// ------------------------------------------------------ edges -> blocks

template <typename IdxT>
__global__ __launch_bounds__(kThreads) void k_edge_count(const IdxT* __restrict__ src,
                                                         const IdxT* __restrict__ dst, int64_t E,
                                                         const int32_t* __restrict__ part, int64_t N,
                                                         int p, const int32_t* __restrict__ lid,
                                                         int64_t n_dst, int32_t* __restrict__ row_cnt,
                                                         unsigned long long* __restrict__ kept,
                                                         int* __restrict__ err)
{
    unsigned long long mine = 0;
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < E;
         e += (int64_t)gridDim.x * kThreads) {
        const int64_t d = (int64_t)dst[e], s = (int64_t)src[e];
        if (d < 0 || d >= N || s < 0 || s >= N) {
            atomicOr(err, 2);
            continue;
        }
        if (part[d] != p) continue;
        atomicAdd(&row_cnt[(int64_t)part[s] * n_dst + lid[d]], 1);
        ++mine;
    }
    // edges kept for this worker, in 64 bits: the 32-bit offsets that follow must not wrap
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(kept, mine);
}

// Uses row_cnt as a countdown cursor: slot order inside a row is arbitrary
// here and fixed by the sort that follows.
template <typename IdxT>
__global__ __launch_bounds__(kThreads) void k_edge_scatter(const IdxT* __restrict__ src,
                                                           const IdxT* __restrict__ dst, int64_t E,
                                                           const int32_t* __restrict__ part,
                                                           int64_t N, int p,
                                                           const int32_t* __restrict__ lid,
                                                           int64_t n_dst, int32_t* __restrict__ row_cnt,
                                                           const int32_t* __restrict__ row_off,
                                                           int32_t* __restrict__ indices_all)
{
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < E;
         e += (int64_t)gridDim.x * kThreads) {
        const int64_t d = (int64_t)dst[e], s = (int64_t)src[e];
        if (d < 0 || d >= N || s < 0 || s >= N) continue;
        if (part[d] != p) continue;
        const int64_t r = (int64_t)part[s] * n_dst + lid[d];
        const int pos = atomicSub(&row_cnt[r], 1) - 1;
        indices_all[(int64_t)row_off[r] + pos] = lid[s];
    }
}

__global__ __launch_bounds__(kThreads) void k_make_indptr(const int32_t* __restrict__ row_off,
                                                          int64_t n_dst, int P,
                                                          int32_t* __restrict__ indptr_all)
{
    const int64_t total = (int64_t)P * (n_dst + 1);
    for (int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x; k < total;
         k += (int64_t)gridDim.x * kThreads) {
        const int64_t q = k / (n_dst + 1), i = k - q * (n_dst + 1);
        indptr_all[k] = row_off[q * n_dst + i] - row_off[q * n_dst];
    }
}

// ------------------------------------------------------------ row sorting

__global__ __launch_bounds__(kThreads) void k_sort_short(const int32_t* __restrict__ off,
                                                         int64_t n_rows, int32_t* __restrict__ data,
                                                         int32_t* __restrict__ long_list,
                                                         int* __restrict__ long_count)
{
    for (int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x; r < n_rows;
         r += (int64_t)gridDim.x * kThreads) {
        const int beg = off[r], len = off[r + 1] - beg;
        if (len <= 1) continue;
        if (len > kShortSort) {
            long_list[atomicAdd(long_count, 1)] = (int32_t)r;
            continue;
        }
        int32_t* a = data + beg;
        for (int k = 1; k < len; ++k) {
            const int32_t x = a[k];
            int m = k - 1;
            while (m >= 0 && a[m] > x) {
                a[m + 1] = a[m];
                --m;
            }
            a[m + 1] = x;
        }
    }
}

// One workgroup per listed row: bitonic network in which every comparator is
// ascending, so the virtual +inf padding behind the row never moves.
__global__ __launch_bounds__(kThreads) void k_sort_long(const int32_t* __restrict__ off,
                                                        int32_t* __restrict__ data,
                                                        const int32_t* __restrict__ long_list,
                                                        const int* __restrict__ long_count)
{
    __shared__ int32_t buf[kLdsSort];
    const int n_list = *long_count;
    for (int w = blockIdx.x; w < n_list; w += gridDim.x) {
        const int64_t r = long_list[w];
        const int beg = off[r], len = off[r + 1] - beg;
        int32_t* g = data + beg;
        const bool in_lds = len <= kLdsSort;
        int32_t* a = in_lds ? buf : g;
        if (in_lds) {
            for (int t = threadIdx.x; t < len; t += kThreads) buf[t] = g[t];
        }
        __syncthreads();
        int n2 = 1;
        while (n2 < len) n2 <<= 1;
        for (int k = 2; k <= n2; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                const bool flip = (j == (k >> 1));
                for (int t = threadIdx.x; t < n2; t += kThreads) {
                    const int partner = flip ? (t ^ (k - 1)) : (t ^ j);
                    if (partner > t && partner < len) {
                        const int32_t x = a[t], y = a[partner];
                        if (x > y) {
                            a[t] = y;
                            a[partner] = x;
                        }
                    }
                }
                __syncthreads();
            }
        }
        if (in_lds) {
            for (int t = threadIdx.x; t < len; t += kThreads) g[t] = buf[t];
        }
        __syncthreads();
    }
}

int sort_rows(const int32_t* off, int64_t n_rows, int32_t* data, int64_t nnz, hipStream_t st,
              DeviceTemps& tmp)
{
    if (n_rows <= 0 || nnz <= 1) return SAR_OK;
    const int64_t cap = nnz / (kShortSort + 1) + 1;
    int32_t* list = nullptr;
    int* count = nullptr;
    SAR_TRY(tmp.alloc(&list, cap));
    SAR_TRY(tmp.alloc(&count, 1));
    SAR_HIP(hipMemsetAsync(count, 0, sizeof(int), st));
    const unsigned g1 = (unsigned)std::min<int64_t>((n_rows + kThreads - 1) / kThreads, 1 << 20);
    k_sort_short<<<g1, kThreads, 0, st>>>(off, n_rows, data, list, count);
    SAR_LAUNCH_CHECK();
    const unsigned g2 = (unsigned)std::min<int64_t>(cap, 16384);
    k_sort_long<<<g2, kThreads, 0, st>>>(off, data, list, count);
    SAR_LAUNCH_CHECK();
    return SAR_OK;
}

// ------------------------------------------------- degree-class row lists

__device__ inline int degree_class(int len) { return len <= 0 ? 0 : 32 - __clz(len); }

__global__ __launch_bounds__(kThreads) void k_class_hist(const int32_t* __restrict__ off, int64_t n,
                                                         int* __restrict__ hist)
{
    __shared__ int h[sar::kNumClasses];
    if (threadIdx.x < sar::kNumClasses) h[threadIdx.x] = 0;
    __syncthreads();
    for (int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x; r < n;
         r += (int64_t)gridDim.x * kThreads) {
        atomicAdd(&h[degree_class(off[r + 1] - off[r])], 1);
    }
    __syncthreads();
    if (threadIdx.x < sar::kNumClasses && h[threadIdx.x]) atomicAdd(&hist[threadIdx.x], h[threadIdx.x]);
}

// cursor[c] starts at the first slot of class c; value written = r | tag.
// Rows without edges (class 0) are listed last, and only if with_empty.
__global__ __launch_bounds__(kThreads) void k_class_place(const int32_t* __restrict__ off, int64_t n,
                                                          int* __restrict__ cursor, uint32_t tag,
                                                          bool with_empty, uint32_t* __restrict__ out)
{
    __shared__ int h[sar::kNumClasses];
    __shared__ int base[sar::kNumClasses];
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (threadIdx.x < sar::kNumClasses) h[threadIdx.x] = 0;
    __syncthreads();
    int c = -1, local = 0;
    if (r < n) {
        c = degree_class(off[r + 1] - off[r]);
        if (c == 0 && !with_empty) c = -1;
        if (c >= 0) local = atomicAdd(&h[c], 1);
    }
    __syncthreads();
    if (threadIdx.x < sar::kNumClasses && h[threadIdx.x])
        base[threadIdx.x] = atomicAdd(&cursor[threadIdx.x], h[threadIdx.x]);
    __syncthreads();
    if (c >= 0) out[base[c] + local] = (uint32_t)r | tag;
}

struct ClassLayout {
    int64_t n_rows = 0, n_long = 0, n_wide = 0;
    int start[sar::kNumClasses];
};

// Degree class from which a list's rows are shared by the four wavefronts of a workgroup: the
// lowest of 128 / 256 / 512 edges (but not below `floor_class`) that leaves them a small minority
// of the list.  A skewed list then has no single-wavefront row long enough to decide when a
// launch ends; a list of uniformly long rows keeps one wavefront per row (no merges).
int pick_long_class(const int* hist, int floor_class)
{
    int64_t n_rows = 0;
    for (int c = 1; c < sar::kNumClasses; ++c) n_rows += hist[c];
    for (int lc = floor_class; lc < sar::kLongClass; ++lc) {
        int64_t n_long = 0;
        for (int c = lc; c < sar::kNumClasses; ++c) n_long += hist[c];
        if (n_long <= std::max<int64_t>(256, n_rows / 16)) return lc;
    }
    return sar::kLongClass;
}

ClassLayout layout_from_hist(const int* hist, int64_t offset, int floor_class)
{
    const int long_class = pick_long_class(hist, floor_class);
    ClassLayout L;
    int64_t run = offset;
    for (int c = sar::kNumClasses - 1; c >= 1; --c) {
        L.start[c] = (int)run;
        run += hist[c];
        L.n_rows += hist[c];
        if (c >= long_class) L.n_long += hist[c];
        if (c > sar::kNarrowMaxClass) L.n_wide += hist[c];
    }
    L.start[0] = (int)run;
    return L;
}

// ------------------------------------- sources of one edge, destination-major

struct SingleTabs {
    const int32_t* t_indptr[SAR_MAX_BLOCKS];
    const int32_t* t_rank[SAR_MAX_BLOCKS];   // null: the source's own id is its row
};

// The entries of the all-blocks index whose source has no other edge in its block, in the order
// of the index (ascending destination, block after block inside a destination): (destination,
// tagged source, row of the source in its block's error).  One wavefront per destination row,
// twice: FILL = false counts a row's entries into cnt[r], FILL = true writes them from off[r] on.
template <bool FILL>
__global__ __launch_bounds__(kThreads) void k_single_list(SingleTabs tabs, const int32_t* __restrict__ f_indptr,
                                                          const uint32_t* __restrict__ f_indices, int64_t n_dst,
                                                          int tag_shift, int32_t* __restrict__ cnt,
                                                          const int32_t* __restrict__ off,
                                                          int32_t* __restrict__ s_dst, uint32_t* __restrict__ s_src,
                                                          int32_t* __restrict__ s_row)
{
    __shared__ const int32_t* ip[SAR_MAX_BLOCKS];
    __shared__ const int32_t* rk[SAR_MAX_BLOCKS];
    if (threadIdx.x < SAR_MAX_BLOCKS) {
        ip[threadIdx.x] = tabs.t_indptr[threadIdx.x];
        rk[threadIdx.x] = tabs.t_rank[threadIdx.x];
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const uint32_t mask = (1u << tag_shift) - 1u;
    const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
    for (int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6); r < n_dst; r += n_waves) {
        const int beg = f_indptr[r], end = f_indptr[r + 1];
        int at = FILL ? off[r] : 0;
        for (int c = beg; c < end; c += 64) {
            uint32_t id = 0;
            int q = 0, j = 0;
            bool single = false;
            if (c + lane < end) {
                id = f_indices[c + lane];
                q = (int)(id >> tag_shift);
                j = (int)(id & mask);
                single = ip[q][j + 1] - ip[q][j] == 1;
            }
            const unsigned long long votes = __ballot(single);
            if (FILL && single) {
                const int mine = at + __popcll(votes & ((1ull << lane) - 1ull));
                s_dst[mine] = (int32_t)r;
                s_src[mine] = id;
                s_row[mine] = rk[q] ? rk[q][j] : j;
            }
            at += __popcll(votes);
        }
        if (!FILL && lane == 0) cnt[r] = at;
    }
}

// --------------------------------------------------- transpose of a block

// One wavefront per listed destination row.
// col_cnt[j] = number of edges of the block whose source is j: one thread per edge
__global__ __launch_bounds__(kThreads) void k_t_count(const int32_t* __restrict__ indices, int64_t nnz,
                                                      int32_t* __restrict__ col_cnt)
{
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * kThreads)
        atomicAdd(&col_cnt[indices[e]], 1);
}

// Destination i of every edge goes into its source's slot range.  LANES lanes share a row of the
// launch list: a whole wavefront for the rows of at least 8 edges at the head of the list, 8 lanes
// for the short rows behind them (most rows of a P-way split have a handful of edges per block).
template <int LANES>
__global__ __launch_bounds__(kThreads) void k_t_scatter(const int32_t* __restrict__ indptr,
                                                        const int32_t* __restrict__ indices,
                                                        const uint32_t* __restrict__ rows,
                                                        int64_t n_rows, int32_t* __restrict__ col_cnt,
                                                        const int32_t* __restrict__ col_off,
                                                        int32_t* __restrict__ t_indices_all)
{
    const int lane = threadIdx.x & (LANES - 1);
    for (int64_t w = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / LANES; w < n_rows;
         w += ((int64_t)gridDim.x * kThreads) / LANES) {
        const int i = (int)rows[w];
        const int beg = indptr[i], end = indptr[i + 1];
        for (int e = beg + lane; e < end; e += LANES) {
            const int j = indices[e];
            const int pos = atomicSub(&col_cnt[j], 1) - 1;
            t_indices_all[(int64_t)col_off[j] + pos] = i;
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_rebase(const int32_t* __restrict__ off, int64_t n_plus_1,
                                                     int32_t* __restrict__ out)
{
    const int32_t base = off[0];
    for (int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x; k < n_plus_1;
         k += (int64_t)gridDim.x * kThreads)
        out[k] = off[k] - base;
}

// flags[j] = 1 if source j has an edge (from global offsets)
__global__ __launch_bounds__(kThreads) void k_nonempty_flags(const int32_t* __restrict__ off, int64_t n,
                                                             int32_t* __restrict__ flags)
{
    for (int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x; k < n;
         k += (int64_t)gridDim.x * kThreads)
        flags[k] = off[k + 1] > off[k] ? 1 : 0;
}

__global__ __launch_bounds__(kThreads) void k_compact(const int32_t* __restrict__ off,
                                                      const int32_t* __restrict__ pos, int64_t n,
                                                      int32_t base_pos, int32_t* __restrict__ out)
{
    for (int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x; k < n;
         k += (int64_t)gridDim.x * kThreads)
        if (off[k + 1] > off[k]) out[pos[k] - base_pos] = (int32_t)k;
}

// ------------------------------------------------- all-blocks (fused) index

struct PtrTable {
    const int32_t* indptr[SAR_MAX_PARTS];     // every handle's blocks (the degree pass), 2 KB of kernel arguments
};

__global__ __launch_bounds__(kThreads) void k_total_degree(PtrTable t, int P, int64_t n_dst,
                                                           int32_t* __restrict__ deg)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i <= n_dst;
         i += (int64_t)gridDim.x * kThreads) {
        int d = 0;
        if (i < n_dst)
            for (int q = 0; q < P; ++q) d += t.indptr[q][i + 1] - t.indptr[q][i];
        deg[i] = d;   // deg[n_dst] = 0 closes the scan
    }
}

struct IdxTable {
    const int32_t* indices[SAR_MAX_BLOCKS];
};

// Row i of the all-blocks index: its sources block after block, tagged with the block.  A
// wavefront takes a row: lane q reads block q's range of the row, then the blocks are copied
// in turn (8 lanes per block range when the blocks are many and the ranges short).
__global__ __launch_bounds__(kThreads) void k_fused_copy(PtrTable t, IdxTable x, int P, int64_t n_dst,
                                                         const int32_t* __restrict__ f_indptr, int tag_shift,
                                                         uint32_t* __restrict__ f_indices)
{
    const int lane = threadIdx.x & 63;
    for (int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6; i < n_dst;
         i += ((int64_t)gridDim.x * kThreads) >> 6) {
        int beg = 0, len = 0;
        if (lane < P) {
            beg = t.indptr[lane][i];
            len = t.indptr[lane][i + 1] - beg;
        }
        int64_t pos = f_indptr[i];
        for (int q = 0; q < P; ++q) {
            const int b = __shfl(beg, q), n = __shfl(len, q);
            for (int e = lane; e < n; e += 64)
                f_indices[pos + e] = (uint32_t)x.indices[q][b + e] | ((uint32_t)q << tag_shift);
            pos += n;
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_check_columns(const int32_t* __restrict__ indptr,
                                                            const int32_t* __restrict__ indices,
                                                            int64_t n_dst, int64_t nnz, int64_t n_src,
                                                            int* __restrict__ err)
{
    for (int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x; k < nnz;
         k += (int64_t)gridDim.x * kThreads)
        if (indices[k] < 0 || indices[k] >= n_src) atomicOr(err, 4);
    for (int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x; k < n_dst;
         k += (int64_t)gridDim.x * kThreads)
        if (indptr[k + 1] < indptr[k]) atomicOr(err, 8);
}

unsigned grid_for(int64_t items, int per_block = kThreads, int64_t cap = 1 << 20)
{
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>((items + per_block - 1) / per_block, cap));
}

template <typename T>
int own(sar_blocks* h, T** out, int64_t count)
{
    void* p = nullptr;
    SAR_HIP(hipMalloc(&p, std::max<int64_t>(count, 1) * sizeof(T)));
    h->owned.push_back(p);
    *out = static_cast<T*>(p);
    return SAR_OK;
}

int bits_for(int64_t n)
{
    int b = 0;
    while (((int64_t)1 << b) < n) ++b;
    return b;
}

// Builds what `flags` asks for on top of per-block CSR arrays already in h->blk.
int derive(sar_blocks* h, hipStream_t st)
{
    const int P = h->P;
    const int64_t n_dst = h->n_dst;
    DeviceTemps tmp;
    if ((h->flags & SAR_BUILD_COMPACT) && !(h->flags & SAR_BUILD_TRANSPOSE))
        return sar::fail(SAR_ERR_INVALID_ARG, "SAR_BUILD_COMPACT needs SAR_BUILD_TRANSPOSE");

    int64_t nnz_total = 0, n_src_total = 0, n_src_max = 0;
    for (auto& b : h->blk) {
        nnz_total += b.nnz;
        n_src_total += b.n_src;
        n_src_max = std::max(n_src_max, b.n_src);
    }
    if (n_src_total >= ((int64_t)1 << 31))
        return sar::fail(SAR_ERR_UNSUPPORTED, "the %d source partitions hold %lld nodes in total; a handle's work "
                         "lists index fewer than 2^31", P, (long long)n_src_total);
    h->tag_shift = std::max(1, bits_for(std::max<int64_t>(n_src_max, 2)));
    if (h->tag_shift + bits_for(P) > 32)
        return sar::fail(SAR_ERR_UNSUPPORTED, "P=%d blocks of up to %lld sources do not fit a 32-bit tagged index",
                         P, (long long)n_src_max);

    PtrTable tab;
    memset(&tab, 0, sizeof(tab));
    for (int q = 0; q < P; ++q) tab.indptr[q] = h->blk[q].indptr;

    // total in-degree |N(i)|
    SAR_TRY(own(h, &h->deg, n_dst + 1));
    k_total_degree<<<grid_for(n_dst + 1), kThreads, 0, st>>>(tab, P, n_dst, h->deg);
    SAR_LAUNCH_CHECK();

    // ---- destination-row launch lists, one per block, longest class first
    int* hist_d = nullptr;
    const int n_hist = (P + 2) * sar::kNumClasses;
    SAR_TRY(tmp.alloc(&hist_d, n_hist));
    SAR_HIP(hipMemsetAsync(hist_d, 0, n_hist * sizeof(int), st));
    for (int q = 0; q < P; ++q) {
        k_class_hist<<<grid_for(n_dst, kThreads, 4096), kThreads, 0, st>>>(h->blk[q].indptr, n_dst,
                                                                           hist_d + q * sar::kNumClasses);
        SAR_LAUNCH_CHECK();
    }
    std::vector<int> hist(n_hist);
    SAR_HIP(hipMemcpyAsync(hist.data(), hist_d, n_hist * sizeof(int), hipMemcpyDeviceToHost, st));
    SAR_HIP(hipStreamSynchronize(st));
    std::vector<int> cursors(n_hist, 0);
    int64_t rows_total = 0;
    std::vector<int64_t> rows_base(P);
    for (int q = 0; q < P; ++q) {
        ClassLayout L = layout_from_hist(&hist[q * sar::kNumClasses], 0, sar::kLongClassBlock);
        h->blk[q].n_rows = L.n_rows;
        h->blk[q].n_long = L.n_long;
        h->blk[q].n_rows_wide = L.n_wide;
        memcpy(&cursors[q * sar::kNumClasses], L.start, sizeof(L.start));
        rows_base[q] = rows_total;
        rows_total += L.n_rows;
    }
    int32_t* rows_all = nullptr;
    SAR_TRY(own(h, &rows_all, rows_total));
    SAR_HIP(hipMemcpyAsync(hist_d, cursors.data(), n_hist * sizeof(int), hipMemcpyHostToDevice, st));
    for (int q = 0; q < P; ++q) {
        h->blk[q].rows = rows_all + rows_base[q];
        k_class_place<<<grid_for(n_dst, kThreads, 1 << 23), kThreads, 0, st>>>(h->blk[q].indptr, n_dst,
                                                            hist_d + q * sar::kNumClasses, 0u, false,
                                                            reinterpret_cast<uint32_t*>(h->blk[q].rows));
        SAR_LAUNCH_CHECK();
    }
    SAR_HIP(hipStreamSynchronize(st));   // cursors (host vector) must outlive the copy

    // ---- all-blocks destination-major index
    if (h->flags & SAR_BUILD_FUSED) {
        if (nnz_total >= ((int64_t)1 << 31))
            return sar::fail(SAR_ERR_UNSUPPORTED, "all-blocks index needs fewer than 2^31 edges, got %lld",
                             (long long)nnz_total);
        SAR_TRY(own(h, &h->f_indptr, n_dst + 1));
        SAR_TRY(exclusive_scan(h->deg, h->f_indptr, n_dst + 1, st, tmp));
        SAR_TRY(own(h, &h->f_indices, nnz_total));
        {
            IdxTable idx;
            memset(&idx, 0, sizeof(idx));
            for (int q = 0; q < P; ++q) idx.indices[q] = h->blk[q].indices;
            k_fused_copy<<<grid_for(n_dst * 64), kThreads, 0, st>>>(tab, idx, P, n_dst, h->f_indptr, h->tag_shift,
                                                                    h->f_indices);
            SAR_LAUNCH_CHECK();
        }
        int* fh = hist_d + P * sar::kNumClasses;
        SAR_HIP(hipMemsetAsync(fh, 0, sar::kNumClasses * sizeof(int), st));
        k_class_hist<<<grid_for(n_dst, kThreads, 4096), kThreads, 0, st>>>(h->f_indptr, n_dst, fh);
        SAR_LAUNCH_CHECK();
        int fhist[sar::kNumClasses];
        SAR_HIP(hipMemcpyAsync(fhist, fh, sizeof(fhist), hipMemcpyDeviceToHost, st));
        SAR_HIP(hipStreamSynchronize(st));
        ClassLayout L = layout_from_hist(fhist, 0, sar::kLongClassBlock);
        h->n_f_rows = L.n_rows;
        h->n_f_long = L.n_long;
        SAR_TRY(own(h, &h->f_rows, n_dst));
        SAR_HIP(hipMemcpyAsync(fh, L.start, sizeof(L.start), hipMemcpyHostToDevice, st));
        k_class_place<<<grid_for(n_dst, kThreads, 1 << 23), kThreads, 0, st>>>(h->f_indptr, n_dst, fh, 0u, true,
                                                            reinterpret_cast<uint32_t*>(h->f_rows));
        SAR_LAUNCH_CHECK();
        SAR_HIP(hipStreamSynchronize(st));
    }

    // ---- source-major transpose of every block
    if (h->flags & SAR_BUILD_TRANSPOSE) {
        if (nnz_total >= ((int64_t)1 << 31))
            return sar::fail(SAR_ERR_UNSUPPORTED, "transpose needs fewer than 2^31 edges in total, got %lld",
                             (long long)nnz_total);
        // counts of all blocks in one array [sum n_src + 1], block q at coff[q]
        std::vector<int64_t> coff(P + 1, 0);
        for (int q = 0; q < P; ++q) coff[q + 1] = coff[q] + h->blk[q].n_src;
        int32_t *col_cnt = nullptr, *col_off = nullptr, *t_indices_all = nullptr, *t_indptr_all = nullptr;
        SAR_TRY(tmp.alloc(&col_cnt, n_src_total + 1));
        SAR_TRY(tmp.alloc(&col_off, n_src_total + 1));
        SAR_HIP(hipMemsetAsync(col_cnt, 0, (n_src_total + 1) * sizeof(int32_t), st));
        for (int q = 0; q < P; ++q) {
            const Block& b = h->blk[q];
            if (b.n_rows == 0) continue;
            k_t_count<<<grid_for(b.nnz, kThreads, 1 << 16), kThreads, 0, st>>>(b.indices, b.nnz, col_cnt + coff[q]);
            SAR_LAUNCH_CHECK();
        }
        SAR_TRY(exclusive_scan(col_cnt, col_off, n_src_total + 1, st, tmp));
        SAR_TRY(own(h, &t_indices_all, nnz_total));
        for (int q = 0; q < P; ++q) {
            const Block& b = h->blk[q];
            if (b.n_rows == 0) continue;
            const uint32_t* rows = reinterpret_cast<const uint32_t*>(b.rows);
            if (b.n_rows_wide > 0) {
                k_t_scatter<64><<<grid_for(b.n_rows_wide * 64), kThreads, 0, st>>>(
                    b.indptr, b.indices, rows, b.n_rows_wide, col_cnt + coff[q], col_off + coff[q], t_indices_all);
                SAR_LAUNCH_CHECK();
            }
            if (b.n_rows > b.n_rows_wide) {
                k_t_scatter<8><<<grid_for((b.n_rows - b.n_rows_wide) * 8), kThreads, 0, st>>>(
                    b.indptr, b.indices, rows + b.n_rows_wide, b.n_rows - b.n_rows_wide, col_cnt + coff[q],
                    col_off + coff[q], t_indices_all);
                SAR_LAUNCH_CHECK();
            }
        }
        SAR_TRY(sort_rows(col_off, n_src_total, t_indices_all, nnz_total, st, tmp));

        // per-block views: own indptr (rebased to the block) and a slice of the indices
        SAR_TRY(own(h, &t_indptr_all, n_src_total + P));
        std::vector<int32_t> block_first(P + 1, 0);
        for (int q = 0; q <= P; ++q)
            SAR_HIP(hipMemcpyAsync(&block_first[q], col_off + coff[q], sizeof(int32_t),
                                   hipMemcpyDeviceToHost, st));
        SAR_HIP(hipStreamSynchronize(st));
        for (int q = 0; q < P; ++q) {
            Block& b = h->blk[q];
            b.t_indptr = t_indptr_all + coff[q] + q;
            b.t_indices = t_indices_all + block_first[q];
            k_rebase<<<grid_for(b.n_src + 1), kThreads, 0, st>>>(col_off + coff[q], b.n_src + 1, b.t_indptr);
            SAR_LAUNCH_CHECK();
        }

        // source launch lists per block + one for all blocks, and the touched lists
        SAR_HIP(hipMemsetAsync(hist_d, 0, n_hist * sizeof(int), st));
        for (int q = 0; q < P; ++q) {
            k_class_hist<<<grid_for(h->blk[q].n_src, kThreads, 4096), kThreads, 0, st>>>(
                h->blk[q].t_indptr, h->blk[q].n_src, hist_d + q * sar::kNumClasses);
            SAR_LAUNCH_CHECK();
        }
        SAR_HIP(hipMemcpyAsync(hist.data(), hist_d, n_hist * sizeof(int), hipMemcpyDeviceToHost, st));
        SAR_HIP(hipStreamSynchronize(st));
        int all_hist[sar::kNumClasses] = {0};
        int64_t t_rows_total = 0;
        std::vector<int64_t> t_base(P);
        for (int q = 0; q < P; ++q) {
            ClassLayout L = layout_from_hist(&hist[q * sar::kNumClasses], 0, sar::kLongClassBlock);
            h->blk[q].n_t_rows = L.n_rows;
            h->blk[q].n_t_long = L.n_long;
            h->blk[q].n_t_wide = L.n_wide;
            memcpy(&cursors[q * sar::kNumClasses], L.start, sizeof(L.start));
            t_base[q] = t_rows_total;
            t_rows_total += L.n_rows;
            for (int c = 0; c < sar::kNumClasses; ++c) all_hist[c] += hist[q * sar::kNumClasses + c];
        }
        ClassLayout LA = layout_from_hist(all_hist, 0, sar::kLongClassBlock);
        h->n_ft_rows = LA.n_rows;
        h->n_ft_long = LA.n_long;
        h->n_ft_wide = LA.n_wide;
        memcpy(&cursors[P * sar::kNumClasses], LA.start, sizeof(LA.start));
        int32_t *t_rows_all = nullptr, *touched_all = nullptr;
        // the launch lists also carry the sources without edges (last), so that the
        // backward kernels write every row of dZ_q; `touched` holds only the others
        SAR_TRY(own(h, &t_rows_all, n_src_total));
        SAR_TRY(own(h, &touched_all, t_rows_total));
        SAR_TRY(own(h, &h->ft_rows, n_src_total));
        SAR_HIP(hipMemcpyAsync(hist_d, cursors.data(), n_hist * sizeof(int), hipMemcpyHostToDevice, st));
        for (int q = 0; q < P; ++q) {
            Block& b = h->blk[q];
            b.t_rows = t_rows_all + coff[q];
            b.touched = touched_all + t_base[q];
            k_class_place<<<grid_for(b.n_src, kThreads, 1 << 23), kThreads, 0, st>>>(b.t_indptr, b.n_src,
                                                                  hist_d + q * sar::kNumClasses, 0u, true,
                                                                  reinterpret_cast<uint32_t*>(b.t_rows));
            SAR_LAUNCH_CHECK();
            k_class_place<<<grid_for(b.n_src, kThreads, 1 << 23), kThreads, 0, st>>>(b.t_indptr, b.n_src,
                                                                  hist_d + P * sar::kNumClasses,
                                                                  (uint32_t)q << h->tag_shift, true, h->ft_rows);
            SAR_LAUNCH_CHECK();
        }
        // touched = ascending ids of the sources with an edge: compaction by scan
        int32_t* pos = nullptr;
        SAR_TRY(tmp.alloc(&pos, n_src_total + 1));
        k_nonempty_flags<<<grid_for(n_src_total), kThreads, 0, st>>>(col_off, n_src_total, pos);
        SAR_LAUNCH_CHECK();
        SAR_HIP(hipMemsetAsync(pos + n_src_total, 0, sizeof(int32_t), st));
        SAR_TRY(exclusive_scan(pos, pos, n_src_total + 1, st, tmp));
        // t_rank[j] = number of touched sources below j, per block (the same scan, rebased)
        int32_t* t_rank_all = nullptr;
        SAR_TRY(own(h, &t_rank_all, n_src_total + P));
        for (int q = 0; q < P; ++q) {
            Block& b = h->blk[q];
            b.t_rank = t_rank_all + coff[q] + q;
            k_rebase<<<grid_for(b.n_src + 1), kThreads, 0, st>>>(pos + coff[q], b.n_src + 1, b.t_rank);
            SAR_LAUNCH_CHECK();
            if (b.n_t_rows == 0) continue;
            k_compact<<<grid_for(b.n_src), kThreads, 0, st>>>(b.t_indptr, pos + coff[q], b.n_src,
                                                              (int32_t)t_base[q], b.touched);
            SAR_LAUNCH_CHECK();
        }
        SAR_HIP(hipStreamSynchronize(st));

        // ---- the sources of one edge, listed from their destinations' side (all-blocks backward):
        // built where they carry at least an eighth of the edges, or on request
        const int64_t n_single = all_hist[1];
        const bool want_singles = (h->flags & SAR_BUILD_SINGLES) ||
                                  (!(h->flags & SAR_BUILD_NO_SINGLES) && n_single * 8 >= nnz_total);
        if ((h->flags & SAR_BUILD_FUSED) && want_singles && n_single > 0) {
            SAR_TRY(own(h, &h->s_dst, n_single));
            SAR_TRY(own(h, &h->s_src, n_single));
            SAR_TRY(own(h, &h->s_row, n_single));
            SingleTabs stabs;
            memset(&stabs, 0, sizeof(stabs));
            for (int q = 0; q < P; ++q) {
                stabs.t_indptr[q] = h->blk[q].t_indptr;
                stabs.t_rank[q] = (h->flags & SAR_BUILD_COMPACT) ? h->blk[q].t_rank : nullptr;
            }
            int32_t *s_cnt = nullptr, *s_off = nullptr;
            SAR_TRY(tmp.alloc(&s_cnt, n_dst + 1));
            SAR_TRY(tmp.alloc(&s_off, n_dst + 1));
            SAR_HIP(hipMemsetAsync(s_cnt + n_dst, 0, sizeof(int32_t), st));
            const unsigned g_list = grid_for(n_dst * 64, kThreads, 1 << 16);
            k_single_list<false><<<g_list, kThreads, 0, st>>>(stabs, h->f_indptr, h->f_indices, n_dst, h->tag_shift,
                                                              s_cnt, nullptr, nullptr, nullptr, nullptr);
            SAR_LAUNCH_CHECK();
            SAR_TRY(exclusive_scan(s_cnt, s_off, n_dst + 1, st, tmp));
            int32_t placed = 0;
            SAR_HIP(hipMemcpyAsync(&placed, s_off + n_dst, sizeof(int32_t), hipMemcpyDeviceToHost, st));
            SAR_HIP(hipStreamSynchronize(st));
            if (placed != n_single)
                return sar::fail(SAR_ERR_STATE, "the all-blocks index lists %d sources of one edge, the transposes %lld",
                                 placed, (long long)n_single);
            k_single_list<true><<<g_list, kThreads, 0, st>>>(stabs, h->f_indptr, h->f_indices, n_dst, h->tag_shift,
                                                             nullptr, s_off, h->s_dst, h->s_src, h->s_row);
            SAR_LAUNCH_CHECK();
            h->n_single = n_single;
        }
    }
    SAR_HIP(hipStreamSynchronize(st));
    return SAR_OK;
}

int check_err_flag(int* err_d, hipStream_t st)
{
    int err = 0;
    SAR_HIP(hipMemcpyAsync(&err, err_d, sizeof(int), hipMemcpyDeviceToHost, st));
    SAR_HIP(hipStreamSynchronize(st));
    if (err & 1) return sar::fail(SAR_ERR_INVALID_ARG, "part[] holds a value outside [0,P)");
    if (err & 2) return sar::fail(SAR_ERR_INVALID_ARG, "edge list holds a node id outside [0,N)");
    if (err & 4) return sar::fail(SAR_ERR_INVALID_ARG, "indices[] holds a column outside [0,n_src)");
    if (err & 8) return sar::fail(SAR_ERR_INVALID_ARG, "indptr[] is not non-decreasing");
    if (err & 16) return sar::fail(SAR_ERR_INVALID_ARG, "dst_ids[] holds a row outside [0,n_dst)");
    return SAR_OK;
}

int build_from_edges(sar_blocks* h, const void* src, const void* dst, int idx_bytes, int64_t E,
                     const int32_t* part, int64_t N, int P, int p, hipStream_t st)
{
    DeviceTemps tmp;
    int* err_d = nullptr;
    SAR_TRY(tmp.alloc(&err_d, 1));
    SAR_HIP(hipMemsetAsync(err_d, 0, sizeof(int), st));

    // 1. rank of every node inside its partition
    const int64_t n_tiles = std::max<int64_t>(1, (N + kPartTile - 1) / kPartTile);
    int32_t *tile_counts = nullptr, *lid = nullptr;
    SAR_TRY(tmp.alloc(&tile_counts, (int64_t)P * n_tiles + 1));
    SAR_TRY(tmp.alloc(&lid, N));
    SAR_HIP(hipMemsetAsync(tile_counts, 0, ((int64_t)P * n_tiles + 1) * sizeof(int32_t), st));
    k_part_tile_count<<<(unsigned)n_tiles, kThreads, 0, st>>>(part, N, P, n_tiles, tile_counts, err_d);
    SAR_LAUNCH_CHECK();
    SAR_TRY(check_err_flag(err_d, st));
    SAR_TRY(exclusive_scan(tile_counts, tile_counts, (int64_t)P * n_tiles + 1, st, tmp));
    std::vector<int32_t> part_first(P + 1);
    for (int q = 0; q <= P; ++q)
        SAR_HIP(hipMemcpyAsync(&part_first[q], tile_counts + (int64_t)q * n_tiles, sizeof(int32_t),
                               hipMemcpyDeviceToHost, st));
    SAR_HIP(hipStreamSynchronize(st));
    k_local_ids<<<(unsigned)n_tiles, kThreads, 0, st>>>(part, N, P, n_tiles, tile_counts, lid);
    SAR_LAUNCH_CHECK();
    const int64_t n_dst = part_first[p + 1] - part_first[p];
    h->n_dst = n_dst;
    h->blk.resize(P);
    for (int q = 0; q < P; ++q) {
        h->blk[q].n_dst = n_dst;
        h->blk[q].n_src = part_first[q + 1] - part_first[q];
    }

    // 2. count, scan, scatter, sort
    const int64_t n_rows_all = (int64_t)P * n_dst;
    int32_t *row_cnt = nullptr, *row_off = nullptr;
    SAR_TRY(tmp.alloc(&row_cnt, n_rows_all + 1));
    SAR_TRY(tmp.alloc(&row_off, n_rows_all + 1));
    SAR_HIP(hipMemsetAsync(row_cnt, 0, (n_rows_all + 1) * sizeof(int32_t), st));
    const unsigned ge = grid_for(E, kThreads, 1 << 16);
    if (E > 0) {
        unsigned long long* kept_d = nullptr;
        SAR_TRY(tmp.alloc(&kept_d, 1));
        SAR_HIP(hipMemsetAsync(kept_d, 0, sizeof(unsigned long long), st));
        if (idx_bytes == 4)
            k_edge_count<int32_t><<<ge, kThreads, 0, st>>>((const int32_t*)src, (const int32_t*)dst, E, part,
                                                           N, p, lid, n_dst, row_cnt, kept_d, err_d);
        else
            k_edge_count<int64_t><<<ge, kThreads, 0, st>>>((const int64_t*)src, (const int64_t*)dst, E, part,
                                                           N, p, lid, n_dst, row_cnt, kept_d, err_d);
        SAR_LAUNCH_CHECK();
        SAR_TRY(check_err_flag(err_d, st));
        unsigned long long kept = 0;
        SAR_HIP(hipMemcpyAsync(&kept, kept_d, sizeof(kept), hipMemcpyDeviceToHost, st));
        SAR_HIP(hipStreamSynchronize(st));
        if (kept >= (1ull << 31))
            return sar::fail(SAR_ERR_UNSUPPORTED, "worker %d's share holds %llu in-edges; a handle holds fewer than 2^31",
                             p, kept);
    }
    SAR_TRY(exclusive_scan(row_cnt, row_off, n_rows_all + 1, st, tmp));
    std::vector<int32_t> block_first(P + 1);
    for (int q = 0; q <= P; ++q)
        SAR_HIP(hipMemcpyAsync(&block_first[q], row_off + (int64_t)q * n_dst, sizeof(int32_t),
                               hipMemcpyDeviceToHost, st));
    SAR_HIP(hipStreamSynchronize(st));
    const int64_t nnz_total = block_first[P];
    int32_t *indices_all = nullptr, *indptr_all = nullptr;
    SAR_TRY(own(h, &indices_all, nnz_total));
    SAR_TRY(own(h, &indptr_all, (int64_t)P * (n_dst + 1)));
    if (E > 0) {
        if (idx_bytes == 4)
            k_edge_scatter<int32_t><<<ge, kThreads, 0, st>>>((const int32_t*)src, (const int32_t*)dst, E,
                                                             part, N, p, lid, n_dst, row_cnt, row_off,
                                                             indices_all);
        else
            k_edge_scatter<int64_t><<<ge, kThreads, 0, st>>>((const int64_t*)src, (const int64_t*)dst, E,
                                                             part, N, p, lid, n_dst, row_cnt, row_off,
                                                             indices_all);
        SAR_LAUNCH_CHECK();
    }
    SAR_TRY(sort_rows(row_off, n_rows_all, indices_all, nnz_total, st, tmp));
    k_make_indptr<<<grid_for((int64_t)P * (n_dst + 1)), kThreads, 0, st>>>(row_off, n_dst, P, indptr_all);
    SAR_LAUNCH_CHECK();
    for (int q = 0; q < P; ++q) {
        h->blk[q].nnz = block_first[q + 1] - block_first[q];
        h->blk[q].indptr = indptr_all + (int64_t)q * (n_dst + 1);
        h->blk[q].indices = indices_all + block_first[q];
    }
    SAR_HIP(hipStreamSynchronize(st));
    return SAR_OK;
}

// ------------------------------------------------ destination subsets

// cnt[r] = length of row ids[r] (0 and an error flag for an id out of range); cnt[n_sub] = 0
__global__ __launch_bounds__(kThreads) void k_subset_count(const int32_t* __restrict__ indptr,
                                                           const int32_t* __restrict__ ids, int64_t n_sub,
                                                           int64_t n_dst, int32_t* __restrict__ cnt, int* err)
{
    for (int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x; r <= n_sub; r += (int64_t)gridDim.x * kThreads) {
        int c = 0;
        if (r < n_sub) {
            const int i = ids[r];
            if (i < 0 || i >= n_dst)
                atomicOr(err, 16);
            else
                c = indptr[i + 1] - indptr[i];
        }
        cnt[r] = c;
    }
}

// new row r = old row ids[r], one wavefront per row
__global__ __launch_bounds__(kThreads) void k_subset_copy(const int32_t* __restrict__ indptr,
                                                          const int32_t* __restrict__ indices,
                                                          const int32_t* __restrict__ ids, int64_t n_sub,
                                                          const int32_t* __restrict__ new_indptr,
                                                          int32_t* __restrict__ new_indices)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * kThreads) >> 6;
    for (int64_t r = wave; r < n_sub; r += n_waves) {
        const int i = ids[r];
        const int beg = indptr[i], len = indptr[i + 1] - beg, at = new_indptr[r];
        for (int k = lane; k < len; k += 64) new_indices[at + k] = indices[beg + k];
    }
}

void destroy(sar_blocks* h)
{
    if (!h) return;
    for (void* p : h->owned) (void)hipFree(p);
    delete h;
}

}  // namespace

namespace {
constexpr int kKnownFlags = SAR_BUILD_TRANSPOSE | SAR_BUILD_FUSED | SAR_BUILD_SKIP_UNTOUCHED | SAR_BUILD_COMPACT |
                            SAR_BUILD_SINGLES | SAR_BUILD_NO_SINGLES;
}

extern "C" int sar_blocks_build(const void* src, const void* dst, int idx_bytes, int64_t E,
                                const int32_t* part, int64_t N, int P, int p, int flags, void* stream,
                                sar_blocks_t** out)
{
    SAR_CHECK_ARG(out != nullptr, "out is null");
    *out = nullptr;
    SAR_CHECK_ARG(idx_bytes == 4 || idx_bytes == 8, "idx_bytes must be 4 or 8, got %d", idx_bytes);
    SAR_CHECK_ARG(E >= 0 && N > 0, "need E >= 0 and N > 0 (E=%lld, N=%lld)", (long long)E, (long long)N);
    SAR_CHECK_ARG(E == 0 || (src && dst), "src/dst is null");
    SAR_CHECK_ARG(part != nullptr, "part is null");
    SAR_CHECK_ARG(P >= 1 && p >= 0 && p < P, "need 0 <= p < P, got p=%d P=%d", p, P);
    SAR_CHECK_ARG((flags & ~kKnownFlags) == 0, "unknown flags 0x%x", flags);
    if (P > SAR_MAX_PARTS)
        return sar::fail(SAR_ERR_UNSUPPORTED, "P=%d exceeds SAR_MAX_PARTS=%d", P, SAR_MAX_PARTS);
    if (P > SAR_MAX_BLOCKS && (flags & SAR_BUILD_FUSED))
        return sar::fail(SAR_ERR_UNSUPPORTED,
                         "P=%d exceeds SAR_MAX_BLOCKS=%d, the most an all-blocks call takes: build without "
                         "SAR_BUILD_FUSED and use the per-block calls", P, SAR_MAX_BLOCKS);
    if (N >= ((int64_t)1 << 31))
        return sar::fail(SAR_ERR_UNSUPPORTED, "N must be below 2^31 (32-bit node ids inside the handle)");
    sar_blocks* h = new (std::nothrow) sar_blocks();
    if (!h) return sar::fail(SAR_ERR_HIP, "out of host memory");
    h->P = P;
    h->flags = flags;
    hipStream_t st = sar::as_stream(stream);
    int rc = build_from_edges(h, src, dst, idx_bytes, E, part, N, P, p, st);
    if (rc == SAR_OK) rc = derive(h, st);
    if (rc != SAR_OK) {
        destroy(h);
        return rc;
    }
    *out = h;
    return SAR_OK;
}

extern "C" int sar_blocks_wrap(int P, int64_t n_dst, const int64_t* n_src, const int32_t* const* indptr,
                               const int32_t* const* indices, int flags, void* stream, sar_blocks_t** out)
{
    SAR_CHECK_ARG(out != nullptr, "out is null");
    *out = nullptr;
    SAR_CHECK_ARG(P >= 1 && n_dst >= 0, "need P >= 1 and n_dst >= 0");
    SAR_CHECK_ARG(n_src && indptr && indices, "n_src/indptr/indices is null");
    SAR_CHECK_ARG((flags & ~kKnownFlags) == 0, "unknown flags 0x%x", flags);
    if (P > SAR_MAX_PARTS)
        return sar::fail(SAR_ERR_UNSUPPORTED, "P=%d exceeds SAR_MAX_PARTS=%d", P, SAR_MAX_PARTS);
    if (P > SAR_MAX_BLOCKS && (flags & SAR_BUILD_FUSED))
        return sar::fail(SAR_ERR_UNSUPPORTED,
                         "P=%d exceeds SAR_MAX_BLOCKS=%d, the most an all-blocks call takes: build without "
                         "SAR_BUILD_FUSED and use the per-block calls", P, SAR_MAX_BLOCKS);
    for (int q = 0; q < P; ++q) {
        SAR_CHECK_ARG(indptr[q] != nullptr, "indptr[%d] is null", q);
        SAR_CHECK_ARG(n_src[q] >= 0 && n_src[q] < ((int64_t)1 << 31), "n_src[%d] out of range", q);
    }
    SAR_CHECK_ARG(n_dst < ((int64_t)1 << 31), "n_dst must be below 2^31");
    hipStream_t st = sar::as_stream(stream);
    sar_blocks* h = new (std::nothrow) sar_blocks();
    if (!h) return sar::fail(SAR_ERR_HIP, "out of host memory");
    h->P = P;
    h->n_dst = n_dst;
    h->flags = flags;
    h->blk.resize(P);
    auto body = [&]() -> int {
        DeviceTemps tmp;
        int* err_d = nullptr;
        SAR_TRY(tmp.alloc(&err_d, 1));
        SAR_HIP(hipMemsetAsync(err_d, 0, sizeof(int), st));
        for (int q = 0; q < P; ++q) {
            Block& b = h->blk[q];
            b.n_dst = n_dst;
            b.n_src = n_src[q];
            b.indptr = indptr[q];
            b.indices = indices[q];
            int32_t ends[2] = {0, 0};
            SAR_HIP(hipMemcpyAsync(&ends[0], indptr[q], sizeof(int32_t), hipMemcpyDeviceToHost, st));
            SAR_HIP(hipMemcpyAsync(&ends[1], indptr[q] + n_dst, sizeof(int32_t), hipMemcpyDeviceToHost, st));
            SAR_HIP(hipStreamSynchronize(st));
            SAR_CHECK_ARG(ends[0] == 0 && ends[1] >= 0, "indptr[%d] must start at 0 and end >= 0", q);
            b.nnz = ends[1];
            SAR_CHECK_ARG(b.nnz == 0 || indices[q] != nullptr, "indices[%d] is null", q);
            k_check_columns<<<grid_for(std::max(b.nnz, n_dst), kThreads, 4096), kThreads, 0, st>>>(
                b.indptr, b.indices, n_dst, b.nnz, b.n_src, err_d);
            SAR_LAUNCH_CHECK();
        }
        SAR_TRY(check_err_flag(err_d, st));
        return derive(h, st);
    };
    int rc = body();
    if (rc != SAR_OK) {
        destroy(h);
        return rc;
    }
    *out = h;
    return SAR_OK;
}

extern "C" int sar_blocks_info(const sar_blocks_t* b, int* P, int64_t* n_dst)
{
    SAR_CHECK_ARG(b != nullptr, "handle is null");
    if (P) *P = b->P;
    if (n_dst) *n_dst = b->n_dst;
    return SAR_OK;
}

extern "C" int sar_blocks_singles(const sar_blocks_t* b, int64_t* n, const int32_t** dst, const uint32_t** src,
                                  const int32_t** row, int* tag_shift)
{
    SAR_CHECK_ARG(b != nullptr && n != nullptr, "handle or n is null");
    *n = b->n_single;
    if (dst) *dst = b->s_dst;
    if (src) *src = b->s_src;
    if (row) *row = b->s_row;
    if (tag_shift) *tag_shift = b->tag_shift;
    return SAR_OK;
}

extern "C" int sar_blocks_get(const sar_blocks_t* b, int q, sar_block_view* v)
{
    SAR_CHECK_ARG(b != nullptr && v != nullptr, "handle or view is null");
    SAR_CHECK_ARG(q >= 0 && q < b->P, "block %d out of range [0,%d)", q, b->P);
    const Block& k = b->blk[q];
    v->n_dst = k.n_dst;
    v->n_src = k.n_src;
    v->nnz = k.nnz;
    v->indptr = k.indptr;
    v->indices = k.indices;
    v->t_indptr = k.t_indptr;
    v->t_indices = k.t_indices;
    v->rows = k.rows;
    v->n_rows = k.n_rows;
    v->n_long = k.n_long;
    v->t_rows = k.t_rows;
    v->n_t_rows = k.n_t_rows;
    v->n_t_long = k.n_t_long;
    v->touched = k.touched;
    v->t_rank = k.t_rank;
    return SAR_OK;
}

extern "C" int sar_blocks_degree(const sar_blocks_t* b, const int32_t** deg)
{
    SAR_CHECK_ARG(b != nullptr && deg != nullptr, "handle or deg is null");
    *deg = b->deg;
    return SAR_OK;
}

extern "C" int sar_blocks_free(sar_blocks_t* b)
{
    destroy(b);
    return SAR_OK;
}

extern "C" int sar_blocks_subset(const sar_blocks_t* b, const int32_t* dst_ids, int64_t n_sub, int flags,
                                 void* stream, sar_blocks_t** out)
{
    SAR_CHECK_ARG(out != nullptr, "out is null");
    *out = nullptr;
    SAR_CHECK_ARG(b != nullptr, "handle is null");
    SAR_CHECK_ARG(n_sub >= 0 && n_sub < ((int64_t)1 << 31), "n_sub must be in [0, 2^31)");
    SAR_CHECK_ARG(n_sub == 0 || dst_ids != nullptr, "dst_ids is null");
    SAR_CHECK_ARG((flags & ~kKnownFlags) == 0, "unknown flags 0x%x", flags);
    hipStream_t st = sar::as_stream(stream);
    sar_blocks* h = new (std::nothrow) sar_blocks();
    if (!h) return sar::fail(SAR_ERR_HIP, "out of host memory");
    h->P = b->P;
    h->n_dst = n_sub;
    h->flags = flags;
    h->blk.resize(b->P);
    auto body = [&]() -> int {
        DeviceTemps tmp;
        int* err_d = nullptr;
        SAR_TRY(tmp.alloc(&err_d, 1));
        SAR_HIP(hipMemsetAsync(err_d, 0, sizeof(int), st));
        for (int q = 0; q < b->P; ++q) {
            const Block& from = b->blk[q];
            Block& to = h->blk[q];
            to.n_dst = n_sub;
            to.n_src = from.n_src;
            int32_t* indptr = nullptr;
            SAR_TRY(own(h, &indptr, n_sub + 1));
            k_subset_count<<<grid_for(n_sub + 1, kThreads, 4096), kThreads, 0, st>>>(from.indptr, dst_ids, n_sub,
                                                                                    b->n_dst, indptr, err_d);
            SAR_LAUNCH_CHECK();
            SAR_TRY(exclusive_scan(indptr, indptr, n_sub + 1, st, tmp));
            int32_t nnz = 0;
            SAR_HIP(hipMemcpyAsync(&nnz, indptr + n_sub, sizeof(int32_t), hipMemcpyDeviceToHost, st));
            SAR_TRY(check_err_flag(err_d, st));      // synchronises; ids are in range beyond this point
            if (nnz < 0) return sar::fail(SAR_ERR_UNSUPPORTED, "block %d of the subset holds 2^31 edges or more", q);
            int32_t* indices = nullptr;
            SAR_TRY(own(h, &indices, nnz));
            if (nnz > 0) {
                k_subset_copy<<<grid_for(n_sub * 64, kThreads, 1 << 16), kThreads, 0, st>>>(
                    from.indptr, from.indices, dst_ids, n_sub, indptr, indices);
                SAR_LAUNCH_CHECK();
            }
            to.indptr = indptr;
            to.indices = indices;
            to.nnz = nnz;
        }
        return derive(h, st);
    };
    int rc = body();
    if (rc != SAR_OK) {
        destroy(h);
        return rc;
    }
    *out = h;
    return SAR_OK;
}
