// Internal declarations shared by the translation units of libsar_mi355x.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/sar_mi355x.h"

namespace sar {

// Records the message for sar_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

#define SAR_HIP(expr)                                                                   \
    do {                                                                                \
        hipError_t sar_e_ = (expr);                                                     \
        if (sar_e_ != hipSuccess)                                                       \
            return ::sar::fail(SAR_ERR_HIP, "%s failed: %s", #expr,                     \
                               hipGetErrorString(sar_e_));                              \
    } while (0)

#define SAR_CHECK_ARG(cond, ...)                                                        \
    do {                                                                                \
        if (!(cond)) return ::sar::fail(SAR_ERR_INVALID_ARG, __VA_ARGS__);              \
    } while (0)

#define SAR_TRY(expr)                                                                   \
    do {                                                                                \
        int sar_rc_ = (expr);                                                           \
        if (sar_rc_ != SAR_OK) return sar_rc_;                                          \
    } while (0)

#define SAR_LAUNCH_CHECK() SAR_HIP(hipGetLastError())

// Rows (or sources) with at least this many edges in a block are "long": they
// are handled by a whole workgroup instead of one wavefront.  A power of two
// so that it coincides with a degree-class boundary.
// Rows the four wavefronts of a workgroup share: those of at least 128, 256 or 512 edges, the
// lowest of the three that leaves them a small minority of their list (chosen per list when it
// is built).  A 300-edge row at the head of one wavefront's share otherwise decides when a
// launch ends (a per-block launch is a dozen rows per wavefront); where nearly all rows are that
// long there is nothing to balance, and sharing them would only add merges.
constexpr int kLongRow = 512;
constexpr int kLongClass = 10;       // 1 + log2(kLongRow)
constexpr int kLongRowBlock = 128;
constexpr int kLongClassBlock = 8;   // 1 + log2(kLongRowBlock)
constexpr int kNumClasses = 32;
// Rows of fewer than 8 edges (degree classes 1..3, and the empty class 0) are
// "narrow": the backward kernels process several of them per wavefront.  (Measured on the
// backward pass of the 8-way products-sized share, fp32: the two kernels together take 3.00 ms
// with the split at 4 edges, 2.92 at 8 and 2.93 at 16; with bf16 rows on the papers-sized share
// the split at 8 and at 16 cost the same.)
constexpr int kNarrowMaxClass = 3;

struct Block {
    int64_t n_dst = 0, n_src = 0, nnz = 0;
    const int32_t* indptr = nullptr;
    const int32_t* indices = nullptr;
    int32_t* t_indptr = nullptr;
    int32_t* t_indices = nullptr;
    int32_t* rows = nullptr;
    int64_t n_rows = 0, n_long = 0;
    int32_t* t_rows = nullptr;
    int64_t n_rows_wide = 0;                             // destination rows with >= 8 edges (head of `rows`)
    int64_t n_t_rows = 0, n_t_long = 0, n_t_wide = 0;   // n_t_wide: sources with >= 8 edges
    int32_t* touched = nullptr;
    int32_t* t_rank = nullptr;                           // [n_src+1]: touched sources below j
};

// Rows of dZ_q / dt_q the backward calls write for a handle with these flags.
inline bool skips_untouched(int flags) { return (flags & (SAR_BUILD_SKIP_UNTOUCHED | SAR_BUILD_COMPACT)) != 0; }

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// score[v,h] = <a[h], Z[v,h]> for one or two vectors a in one pass over Z (gat.hip).
int gat_scores2(const void* Z, int dtype, int64_t n, int H, int D, const float* a, float* score,
                const float* a2, float* score2, void* stream);

}  // namespace sar

struct sar_blocks {
    int P = 0;
    int64_t n_dst = 0;
    int flags = 0;
    std::vector<sar::Block> blk;
    int32_t* deg = nullptr;
    // All-blocks destination-major index: row i lists its sources block after
    // block (q ascending), each entry (q << tag_shift) | local source id.
    int32_t* f_indptr = nullptr;   // [n_dst+1]
    uint32_t* f_indices = nullptr; // [sum nnz]
    int32_t* f_rows = nullptr;     // destinations with deg > 0, longest class first
    int64_t n_f_rows = 0, n_f_long = 0;
    int tag_shift = 0;
    // All-blocks source-side work list: (q << tag_shift) | local source id of
    // every source with an edge, longest class first.
    uint32_t* ft_rows = nullptr;
    int64_t n_ft_rows = 0, n_ft_long = 0, n_ft_wide = 0;
    // The sources that have ONE edge in their block (the last n_single entries of ft_rows that
    // have an edge), listed in the order of that edge's destination: destination, tagged source,
    // row of the source in its block's error.  Null / 0 where the list was not built.
    int32_t* s_dst = nullptr;
    uint32_t* s_src = nullptr;
    int32_t* s_row = nullptr;
    int64_t n_single = 0;
    std::vector<void*> owned;      // device allocations freed with the handle
};
