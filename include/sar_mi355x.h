/*
 * sar_mi355x.h -- C ABI of the SAR aggregation hot path for AMD MI355X (gfx950).
 *
 * What the library computes (arXiv 2111.06483): one worker p's sequential
 * aggregation of its destination partition V_p over P source-partition edge
 * blocks G_{p,q} (Sec. 3.2, Alg. 1), the per-block backward of Alg. 2, with
 *   - sum / mean aggregation of neighbour features (Eq. 2),
 *   - the fused, rematerialising attention kernels of Sec. 3.3 for GAT
 *     (Eq. 3) using the running-maximum incremental softmax of Sec. 3.4,
 *   - the node-wise transform z = W h of Eq. 1, written row-major as Z = X W.
 *
 * Conventions that hold for every call
 *   - Every function returns 0 (SAR_OK) or a negative sar_status.  The text of
 *     the most recent failure on the calling thread: sar_last_error().
 *     No C++ exception crosses this boundary.
 *   - Unless a parameter says "host", every pointer is a DEVICE pointer on the
 *     current HIP device, allocated and owned by the caller.  The library keeps
 *     no reference to caller memory after a call returns, except that a handle
 *     made by sar_blocks_wrap() borrows the CSR arrays it was given.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Compute calls only enqueue work on it and return; they do not
 *     synchronise.  sar_blocks_build / sar_blocks_wrap allocate device memory
 *     and synchronise the stream before returning.
 *   - An edge j->i carries a message from source j to destination i.  Rows of
 *     a block are destinations (ids local to V_p), columns are sources (ids
 *     local to V_q).  Local id = rank of the global id among the nodes of the
 *     same partition, ascending.
 *   - Feature tensors are row-major [n, H, D] (F = H*D contiguous values per
 *     node; heads are independent and concatenated).  `dtype` selects their
 *     storage: SAR_F32 or SAR_BF16 (round-to-nearest-even on store).  All
 *     running state, scores, log-sum-exps and parameter gradients are fp32 and
 *     all accumulation is fp32.
 *   - a_r multiplies the destination's z_i and a_l the source's z_j: the vector
 *     a of Eq. 3 is [a_r ; a_l] in the order the equation writes z_i || z_j.
 *   - Shapes.  A wavefront covers a head with 64 lanes that each move the largest
 *     piece of 16, 8, 4 (or, for bf16, 2) bytes that divides the head: every head
 *     width is accepted as long as the head fits 64 such lanes (any D up to 256 that
 *     is a multiple of 4; else fp32: D <= 128 for even D, D <= 64 for odd D; bf16:
 *     D <= 128 for even D, D <= 64 for odd D).  A wider head returns
 *     SAR_ERR_UNSUPPORTED.  Rows of several heads are processed as several launches
 *     over groups of heads, rows of the sum/mean calls (any F) over column ranges.
 *     The fastest kernels take head widths that are a multiple of 4 in layers of
 *     1, 2, 4, 8 heads or a multiple thereof (4 x 64, 8 x 32, 4 x 32, 2 x 100, ...);
 *     the results do not depend on which kernel a shape takes.
 *   - A destination with no in-edge at all has out = 0 and L = -inf, and
 *     contributes nothing to any gradient; the mean of an empty set is 0.
 *     A tensor without elements (n_dst = 0, or a block without sources) may be
 *     passed as NULL; the backward calls still write the zero rows of dZ_q.
 *   - A repeated edge counts with its multiplicity (one softmax term / one
 *     summand / one unit of degree per copy).
 */
#ifndef SAR_MI355X_H
#define SAR_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SAR_OK = 0,
    SAR_ERR_INVALID_ARG = -1, /* null pointer, negative size, id out of range ... */
    SAR_ERR_UNSUPPORTED = -2, /* dtype / H / D / P combination the kernels do not cover */
    SAR_ERR_HIP = -3,         /* a HIP runtime call failed (text has hipGetErrorString) */
    SAR_ERR_STATE = -4        /* handle lacks what the call needs (e.g. no transpose) */
} sar_status;

typedef enum { SAR_F32 = 0, SAR_BF16 = 1 } sar_dtype;

/* The non-linearity sigma of Eq. 2 / Eq. 3.  The paper leaves sigma open; ReLU is
 * the one offered, its derivative being a function of the output alone. */
typedef enum { SAR_ACT_NONE = 0, SAR_ACT_RELU = 1 } sar_act;

/* Most blocks one batched (..._all) call can take, hence most partitions of a handle built with
 * SAR_BUILD_FUSED; and most partitions of any handle.  A handle of more than SAR_MAX_BLOCKS
 * partitions (the paper's runs go up to 128 workers) is built without SAR_BUILD_FUSED and used
 * block by block, which is the streaming form of Alg. 1 / Alg. 2 anyway. */
#define SAR_MAX_BLOCKS 64
#define SAR_MAX_PARTS 256

/* flags of sar_blocks_build / sar_blocks_wrap */
#define SAR_BUILD_TRANSPOSE 1 /* also build the source-major index (needed by every *_bwd_*) */
#define SAR_BUILD_FUSED 2     /* also build the all-blocks row index (needed by every *_all) */
/* Backward passes skip the sources that have no edge in a block: their rows of dZ_q (and dt_q)
 * are NOT written.  A worker exchanges only the rows V_{p,q} of a partition that its
 * destinations read (Sec. 3.2), so the error E_{p->q} has no other rows; with full-height
 * buffers zero them once, the skipped rows never change (the handle's `touched` lists name
 * the others).  Without this flag every row of dZ_q, dt_q is written (zeros where no edge). */
#define SAR_BUILD_SKIP_UNTOUCHED 4
/* The error E_{p->q} in the shape it is exchanged in (Alg. 2: worker p sends worker q the errors
 * of the rows V_{p,q} it fetched, nothing else): every backward call on the handle takes dZ_q
 * (and dt_q) with n_t_rows rows instead of n_src, row r belonging to source touched[r]
 * (ascending local id).  Neither zero rows are written nor has a consumer to skip them; the
 * receiver adds row r to its row touched[r] (t_rank gives the inverse map).  Needs
 * SAR_BUILD_TRANSPOSE; implies that sources without an edge get nothing written. */
#define SAR_BUILD_COMPACT 8
/* Sources that have ONE edge in their block.  The backward pass of Alg. 2 walks a block from its
 * sources' side; a source of one edge then costs its own row, its error row and a gathered row of
 * the upstream error with that destination's record.  Walked from the destination's side the same
 * edge costs the source's row and one write of its error row, and nobody else writes that row.
 * A handle with TRANSPOSE and FUSED lists those sources destination-major (sar_blocks_singles)
 * when they carry at least an eighth of the worker's edges, always with SAR_BUILD_SINGLES, never
 * with SAR_BUILD_NO_SINGLES; sar_gat_bwd_all takes them from that list where it exists.  Results
 * are the same either way up to the order of fp32 sums. */
#define SAR_BUILD_SINGLES 16
#define SAR_BUILD_NO_SINGLES 32

typedef struct sar_blocks sar_blocks_t; /* opaque, library-owned */

/* One block G_{p,q} = (V_{p,q}, E_{p,q}) (Sec. 3.2) as seen by the caller.
 * All pointers are device pointers borrowed from the handle; they die with it.
 *   indptr/indices      destination-major CSR: sources of row i are
 *                       indices[indptr[i] .. indptr[i+1]), ascending, local to V_q
 *   t_indptr/t_indices  the same edges source-major: destinations of source j,
 *                       ascending, local to V_p          (NULL without TRANSPOSE)
 *   rows / t_rows       the n_rows rows (resp. n_t_rows sources) that have at
 *                       least one edge in this block, ordered longest-first by
 *                       degree class: the launch order of the kernels.  The
 *                       first n_long (resp. n_t_long) of them have at least 128
 *                       edges (256 or 512 where rows that long are more than a
 *                       sixteenth of the list).  The order inside a degree class is unspecified.
 *                       t_rows continues with the n_src - n_t_rows sources that
 *                       have no edge (the backward kernels zero their rows).
 *   touched             = t_rows sorted ascending: V_{p,q} intersected with V_q,
 *                       the rows of Z_q a remote fetch would have to carry
 *                       (Alg. 1, "Fetch Z_{q->p}")        (NULL without TRANSPOSE)
 *   t_rank              [n_src+1]: t_rank[j] = number of entries of touched below j, so
 *                       touched[t_rank[j]] == j exactly when t_rank[j+1] > t_rank[j]: the
 *                       row of a compact dZ_q that belongs to source j
 *                                                          (NULL without TRANSPOSE)
 */
typedef struct {
    int64_t n_dst, n_src, nnz;
    const int32_t* indptr;
    const int32_t* indices;
    const int32_t* t_indptr;
    const int32_t* t_indices;
    const int32_t* rows;
    int64_t n_rows, n_long;
    const int32_t* t_rows;
    int64_t n_t_rows, n_t_long;
    const int32_t* touched;
    const int32_t* t_rank;
} sar_block_view;

/* Text of the last error on this thread ("" if none).  Host pointer, valid until
 * the next failing call on the same thread. */
const char* sar_last_error(void);

/* ABI version of this header (currently 5). */
int sar_version(void);

/* ------------------------------------------------------------------ blocks
 * Sec. 3.2: worker p holds one subgraph per source partition q; its edge set
 * E_{p,q} is every edge that starts in partition q and ends in partition p.
 */

/* Build worker p's P blocks from a global edge list.
 *   src,dst    [E] global node ids of the edges j->i (src = j, dst = i);
 *              idx_bytes = 4 (int32) or 8 (int64).  Edges whose destination is
 *              not in partition p are ignored.  Ids must lie in [0,N).
 *              E is not limited (the whole graph's list may be passed); the edges
 *              KEPT for worker p must be fewer than 2^31 (32-bit offsets inside
 *              the handle), else SAR_ERR_UNSUPPORTED.
 *   part       [N] partition of every node, each in [0,P)
 *   P <= SAR_MAX_PARTS (<= SAR_MAX_BLOCKS with SAR_BUILD_FUSED), N < 2^31.
 * The CSR arrays, their transposes, the degrees and the touched lists / ranks are
 * integer work and bit-exact: they do not depend on thread scheduling.  The launch
 * lists (rows, t_rows) are filled through atomic cursors, so the order of the rows
 * INSIDE a degree class differs from build to build; that order decides which
 * workgroup sums which rows into the partial sums of da_l / da_r, whose last bits
 * are therefore reproducible for one handle, not across handles built from the same
 * edges (ds is order-dependent through its atomics in any case).
 * *out is a new handle the caller frees with sar_blocks_free. */
int sar_blocks_build(const void* src, const void* dst, int idx_bytes, int64_t E,
                     const int32_t* part, int64_t N, int P, int p, int flags, void* stream,
                     sar_blocks_t** out);

/* Wrap P caller-built destination-major CSR blocks (device arrays, borrowed
 * until sar_blocks_free) and build the derived indexes `flags` asks for.
 *   n_src      host [P], indptr host [P] of device int32 [n_dst+1],
 *   indices    host [P] of device int32 [nnz_q]; columns must be < n_src[q].
 * Rows need not be sorted for the kernels to be correct. */
int sar_blocks_wrap(int P, int64_t n_dst, const int64_t* n_src, const int32_t* const* indptr,
                    const int32_t* const* indices, int flags, void* stream, sar_blocks_t** out);

/* Blocks restricted to the destinations a layer's output is needed for (the
 * message flow graphs of App. B: only the nodes that can influence a labelled
 * output are updated at each layer).  Row r of every block of the new handle
 * is row dst_ids[r] of b (device int32 [n_sub], each in [0, n_dst), any order;
 * a repeated id gives a repeated row); sources keep their local ids, so Z_q,
 * dZ_q keep their shapes and the new handle's `touched` lists name the source
 * rows the previous layer has to produce.  Destination-side tensors of calls
 * on the new handle have n_sub rows.  The new handle owns its arrays and is
 * independent of b; free it with sar_blocks_free. */
int sar_blocks_subset(const sar_blocks_t* b, const int32_t* dst_ids, int64_t n_sub, int flags,
                      void* stream, sar_blocks_t** out);

/* *P = number of blocks, *n_dst = |V_p|. */
int sar_blocks_info(const sar_blocks_t* b, int* P, int64_t* n_dst);

/* Fill *v (host struct) with block q's device pointers and sizes. */
int sar_blocks_get(const sar_blocks_t* b, int q, sar_block_view* v);

/* The handle's destination-major list of the sources that have one edge in their block (Alg. 2
 * walked from the destination for them; see SAR_BUILD_SINGLES): *n entries, entry e being the edge
 * into destination dst[e] from source src[e] = (q << *tag_shift) | j, whose row in block q's error
 * E_{p->q} is row[e] (its rank among the touched sources with SAR_BUILD_COMPACT, else j).  The
 * order is that of the all-blocks index: ascending destination, inside a destination ascending
 * block, inside a block ascending source (integer work, bit-exact like the other index arrays).
 * *n = 0 and null arrays where the list was not built.  Device pointers borrowed from the
 * handle; any of dst, src, row, tag_shift may be NULL. */
int sar_blocks_singles(const sar_blocks_t* b, int64_t* n, const int32_t** dst, const uint32_t** src,
                       const int32_t** row, int* tag_shift);

/* *deg = device int32 [n_dst]: total in-degree |N(i)| over all blocks (Eq. 2). */
int sar_blocks_degree(const sar_blocks_t* b, const int32_t** deg);

/* Free the handle and everything the library allocated for it. */
int sar_blocks_free(sar_blocks_t* b);

/* ------------------------------------------------------- Eq. 2: sum / mean
 * Alg. 1 with m_{j->i} = z_j:  Acc_i += sum over the block's edges of z_j.
 */

/* acc[i,:] += sum_{(j->i) in block q} Zq[j,:].   acc fp32 [n_dst,F] in/out
 * (zero it before the first block); Zq [n_src_q,F] of `dtype`. */
int sar_spmm_block(const sar_blocks_t* b, int q, const void* Zq, int dtype, int F, float* acc,
                   void* stream);

/* After the last block: agg = acc (mean == 0) or acc / |N(i)| (Eq. 2; 0 when
 * |N(i)| = 0), then the node update of Eq. 2, out = act(agg + residual).
 * residual [n_dst,F] of `dtype` holds the rows W_res h_i (e.g. from
 * sar_linear_fwd) or is NULL (= 0); act is SAR_ACT_*.  With residual = NULL and
 * act = SAR_ACT_NONE out is the plain aggregate.  out [n_dst,F] of `dtype`
 * (may alias residual); deg from sar_blocks_degree. */
int sar_spmm_end(const int32_t* deg, int mean, const float* acc, const void* residual, int act,
                 void* out, int dtype, int64_t n_dst, int F, void* stream);

/* All P blocks in one launch, the accumulator never leaving registers; same
 * result as P sar_spmm_block calls in block order followed by sar_spmm_end.
 * Zq: host array [P] of device pointers.  Needs SAR_BUILD_FUSED. */
int sar_spmm_all(const sar_blocks_t* b, const void* const* Zq, int dtype, int F, int mean,
                 const void* residual, int act, void* out, void* stream);

/* Backward through the non-linearity of Eq. 2 / Eq. 3, with its derivative
 * taken from the output: G = dH * act'(.), for ReLU G = dH where h > 0, else 0.
 * h, dH, G: `count` values of `dtype` (16-byte aligned; G may alias dH).  G is then the error of the aggregate
 * (for sar_spmm_bwd_block) and of the residual rows (for sar_linear_bwd). */
int sar_act_bwd(const void* h, const void* dH, int act, void* G, int dtype, int64_t count,
                void* stream);

/* Case 1 of Sec. 3.2 (the gradient of a sum does not need the features):
 * dZq[j,:] = sum_{(j->i) in block q} G[i,:] / (mean ? |N(i)| : 1).
 * dZq [n_src_q,F] of `dtype` is OVERWRITTEN (it is the error E_{p->q} of
 * Alg. 2); on a SAR_BUILD_COMPACT handle it has n_t_rows rows, in `touched` order.
 * G [n_dst,F] of `dtype`.  Needs SAR_BUILD_TRANSPOSE. */
int sar_spmm_bwd_block(const sar_blocks_t* b, int q, const void* G, int mean, int dtype, int F,
                       void* dZq, void* stream);

/* The same for all P blocks in one launch (same results as P
 * sar_spmm_bwd_block calls).  dZq: host array [P] of device pointers. */
int sar_spmm_bwd_all(const sar_blocks_t* b, const void* G, int mean, int dtype, int F,
                     void* const* dZq, void* stream);

/* The owner's side of Alg. 2's error exchange (E_p = sum over workers q of E_{q->p}) for one
 * received compact error: Ep[i,:] (+)= Eq[t_rank[i],:] for every row i that has a row in Eq
 * (t_rank[i+1] > t_rank[i]); the other rows are left alone (accumulate != 0) or set to zero
 * (accumulate == 0, which turns a compact error into a full-height one).
 *   Eq      [n_t_rows, F] of `dtype`: dZ_q of a SAR_BUILD_COMPACT handle (may be NULL when no
 *           row of the block is touched)
 *   t_rank  device int32 [n+1]: the t_rank of the block the error came from (sar_block_view)
 *   Ep      [n, F] of `dtype`, n = that block's n_src; must not alias Eq */
int sar_error_add(const void* Eq, const int32_t* t_rank, int accumulate, void* Ep, int dtype, int64_t n,
                  int F, void* stream);

/* ------------------------------------------------------ Eq. 3: attention
 * e_{j->i} = LeakyReLU(a^T (z_i || z_j)) = LeakyReLU(s_i + t_j) per head with
 * s = <a_r, z_i>, t = <a_l, z_j>;  out_i = sum_j softmax_j(e_{j->i}) z_j.
 */

/* score[v,h] = <a[h,:], Z[v,h,:]>.  Z [n,H,D] of `dtype`, a fp32 [H,D],
 * score fp32 [n,H].  Used for s (a = a_r, Z = Z_dst) and t_q (a = a_l, Z = Z_q). */
int sar_gat_scores(const void* Z, int dtype, int64_t n, int H, int D, const float* a,
                   float* score, void* stream);

/* Start of Alg. 1's loop: running state of Sec. 3.4, m = -inf, l = 0, acc = 0.
 * m,l fp32 [n_dst,H]; acc fp32 [n_dst,H,D]. */
int sar_gat_fwd_begin(float* m, float* l, float* acc, int64_t n_dst, int H, int D, void* stream);

/* One block of Alg. 1 with the fused kernel of Sec. 3.3: for every destination
 * with an edge in block q, per head: new running maximum m' = max(m, max_j e),
 * l = l exp(m-m') + sum_j exp(e-m'), acc = acc exp(m-m') + sum_j exp(e-m') z_j.
 * No per-edge value is written to memory.  Destinations without an edge in the
 * block are not touched.  s fp32 [n_dst,H].  The source halves come either
 * from tq (fp32 [n_src_q,H], e.g. shipped along with Z_q by its owner) or, when
 * tq is NULL, are formed inside the kernel from a_l (fp32 [H,D], 16-byte
 * aligned) and each gathered row, which saves the separate pass over Z_q. */
int sar_gat_fwd_block(const sar_blocks_t* b, int q, const void* Zq, const float* s,
                      const float* tq, const float* a_l, int dtype, int H, int D, float slope,
                      float* m, float* l, float* acc, void* stream);

/* After the last block: out = act(acc / l) (the division of Sec. 3.2 and the
 * non-linearity of Eq. 3; act = SAR_ACT_NONE leaves the aggregate as it is),
 * and the log-sum-exp L = m + log l that the backward pass reads.
 * out [n_dst,H,D] of `dtype`, L fp32 [n_dst,H]. */
int sar_gat_fwd_end(const float* m, const float* l, const float* acc, int act, void* out, float* L,
                    int dtype, int64_t n_dst, int H, int D, void* stream);

/* All P blocks in one launch: each destination walks its blocks in order
 * q = 0..P-1 with the same running-maximum updates, state in registers.
 * Zq, tq: host arrays [P] of device pointers; tq may be NULL (then a_l is used
 * as in sar_gat_fwd_block).  Needs SAR_BUILD_FUSED. */
int sar_gat_fwd_all(const sar_blocks_t* b, const void* const* Zq, const float* s,
                    const float* const* tq, const float* a_l, int dtype, int H, int D, float slope,
                    int act, void* out, float* L, void* stream);

/* Bytes of scratch the backward calls below need for these sizes. */
int sar_gat_workspace_bytes(int64_t n_dst, int64_t n_src_max, int H, int D, size_t* bytes);

/* Start of Alg. 2's loop.  Packs what the backward kernel needs per destination
 * and head into one 16-byte record rec[i,h] = (s log2(e), L log2(e), delta, 0)
 * with delta[i,h] = <G[i,h,:], out[i,h,:]>, and sets ds = 0.
 * G (the error e_Acc) and out [n_dst,H,D] of `dtype`; s, L fp32 [n_dst,H] (from
 * the forward pass); rec fp32 [n_dst,H,4] (16-byte aligned); ds fp32 [n_dst,H].
 * When the forward pass applied a non-linearity (act != SAR_ACT_NONE), out is
 * its output h and G the error of h; the error of the aggregate, G * act'(.),
 * is written to Gact ([n_dst,H,D] of `dtype`, may alias G) and it is Gact that
 * the block calls below take as their G.  With SAR_ACT_NONE Gact is not used
 * and may be NULL. */
int sar_gat_bwd_begin(const void* G, const void* out, const float* s, const float* L, int act,
                      void* Gact, int dtype, float* rec, float* ds, int64_t n_dst, int H, int D,
                      void* stream);

/* One block of Alg. 2 with the rematerialising kernel of Sec. 3.3.  For every
 * edge the coefficient alpha = exp(e - L_i) is recomputed from s_i, t_j, L_i:
 *   de = alpha (<G_i, z_j> - delta_i),  du = de * (1 if s_i+t_j > 0 else slope)
 *   dZq[j] = sum_i alpha G_i + dtq[j] a_l     (OVERWRITTEN: the error E_{p->q})
 *   dtq[j] = sum_i du                          (OVERWRITTEN, fp32 [n_src_q,H])
 *   ds[i] += du                                (accumulates over blocks; atomic,
 *                                               so its rounding order may vary)
 *   da_l  += sum_j dtq[j] Zq[j]                (accumulates over blocks, fp32 [H,D])
 * The kernel walks the source-major index (needs SAR_BUILD_TRANSPOSE): every
 * source gathers its destinations' G rows, so dZq is written once, without
 * atomics.  rec from sar_gat_bwd_begin; tq may be NULL, then t_j = <a_l, z_j> is
 * formed from the row the wavefront owns; a_l 16-byte aligned; work: scratch of
 * at least sar_gat_workspace_bytes, 16-byte aligned.  On a SAR_BUILD_COMPACT handle dZq and
 * dtq have n_t_rows rows, row r for source touched[r]; Zq and tq stay full height.
 * dtq may be NULL: the per-source sums are an intermediate (both of their uses, dtq[j] a_l in
 * dZq and the sum into da_l, happen inside the kernel) and are then not written. */
int sar_gat_bwd_block(const sar_blocks_t* b, int q, const void* Zq, const void* G, const float* tq,
                      const float* rec, const float* a_l, int dtype, int H, int D, float slope,
                      void* dZq, float* dtq, float* ds, float* da_l, void* work, size_t work_bytes,
                      void* stream);

/* All P blocks of Alg. 2's loop in one launch (same results as P
 * sar_gat_bwd_block calls).  Zq, tq, dZq, dtq: host arrays [P] of device
 * pointers; dtq may be NULL as a whole (see sar_gat_bwd_block).  Needs SAR_BUILD_TRANSPOSE. */
int sar_gat_bwd_all(const sar_blocks_t* b, const void* const* Zq, const void* G,
                    const float* const* tq, const float* rec, const float* a_l, int dtype, int H,
                    int D, float slope, void* const* dZq, float* const* dtq, float* ds, float* da_l,
                    void* work, size_t work_bytes, void* stream);

/* After the last block, the destination side of the score:
 * dZdst[i] = ds[i] a_r + dZadd[i] (OVERWRITTEN, `dtype`), da_r += sum_i ds[i] Zdst[i].
 * dZadd may be NULL (= 0); a worker passes its local block's dZq here to get
 * the whole error of its own rows, E_{p->p} plus the destination-score term,
 * in one tensor for Z_p.backward.  dZadd may alias dZdst.
 * dZadd_rank: NULL when dZadd has one row per destination.  For a COMPACT dZadd (the local
 * block's dZq of a SAR_BUILD_COMPACT handle) pass that block's t_rank (device int32
 * [n_dst+1]): row i then receives dZadd[dZadd_rank[i]] if dZadd_rank[i+1] > dZadd_rank[i]
 * and nothing otherwise; such a dZadd must not alias dZdst.
 * dZdst may be NULL when the error is not wanted as a tensor (sar_linear_bwd_rows forms it
 * inside Z_p.backward): then only da_r is produced and dZadd is not read. */
int sar_gat_bwd_end(const void* Zdst, const float* ds, const float* a_r, const void* dZadd,
                    const int32_t* dZadd_rank, void* dZdst, float* da_r, int dtype, int64_t n_dst, int H,
                    int D, void* work, size_t work_bytes, void* stream);

/* sar_gat_bwd_end for callers that cannot allocate device memory or take a workspace
 * along: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and the same results as sar_gat_bwd_end,
 * but the per-workgroup partial sums of da_r live in a 4 MiB array that is part of the
 * library's device image (one copy per GPU, held until the process ends) instead of a
 * caller workspace.  The call allocates nothing and frees nothing.  Limit: a launch
 * needs (workgroups x values per head group) <= 2048 x 512 partial sums, which every
 * shape the library supports satisfies; anything beyond returns SAR_ERR_UNSUPPORTED.
 * All calls on one GPU share that array and it keeps the last call's contents (every
 * call overwrites the part it reads, nothing has to start at zero): two calls that
 * overlap in time on the same GPU -- different streams or threads -- race; serialise
 * them.  The first call on a device looks up the array's device address (no allocation);
 * make that call outside graph capture. */
int sar_gat_bwd_end_noalloc(const void* Zdst, const float* ds, const float* a_r, const void* dZadd,
                            const int32_t* dZadd_rank, void* dZdst, float* da_r, int dtype, int64_t n_dst,
                            int H, int D, void* stream);

/* ------------------------------------------------- Eq. 1: Z = X W on MFMA */

/* Z[n,F] = X[n,K] W[K,F]; X, Z of `dtype`, W fp32 row-major.  When a_score is
 * non-null (fp32 [H,D], F = H*D) also writes score[v,h] = <a_score[h], Z[v,h]>
 * from the fp32 accumulators (fp32 [n,H]); a second pair (a_score2, score2)
 * may be given as well.  Pass H = D = 0 and null pointers for no scores. */
int sar_linear_fwd(const void* X, const float* W, void* Z, int dtype, int64_t n, int K, int F,
                   int H, int D, const float* a_score, float* score, const float* a_score2,
                   float* score2, void* stream);

/* What Z.backward(E) of Alg. 2 does for the transform: dW += X^T dZ (fp32
 * [K,F], accumulates so that several blocks can add up), dX = dZ W^T
 * (OVERWRITTEN, `dtype`, may be NULL to skip).  work: scratch of at least
 * sar_linear_workspace_bytes. */
int sar_linear_bwd(const void* X, const void* dZ, const float* W, float* dW, void* dX, int dtype,
                   int64_t n, int K, int F, void* work, size_t work_bytes, void* stream);

/* Z_p.backward(E_p) of Alg. 2 (the step "Z.backward(E)" after the errors have been summed)
 * without E_p ever being stored:  dW += X^T E_p,  dX = E_p W^T  with
 *     E_p[i,h,:] = E[r(i),h,:] + ds[i,h] a_r[h,:]        (F = H*D values per row),
 * the rows of E_p formed in fp32 where the two products load them and rounded to `dtype`
 * as a stored E_p would have been: the results equal, bit for bit, those of
 * sar_gat_bwd_end (or sar_error_add) into a tensor followed by sar_linear_bwd on it.
 *   E       [n_E,F] of `dtype`: the stored part; NULL with n_E = 0 when there is none (a
 *           compact error of a block without edges, or a layer with the score term only).
 *   E_rank  NULL: E has one row per node (n_E = n).  Otherwise device int32 [n+1], the
 *           t_rank of a SAR_BUILD_COMPACT handle: node i's row is E[E_rank[i]] if
 *           E_rank[i+1] > E_rank[i], and zero otherwise (E_{p->p} of the local block).
 *   ds, a_r [n,H] and [H,D] fp32, both or neither: the destination-score term of the
 *           attention layer (what sar_gat_bwd_end would add); NULL for a layer without it.
 *   rows    NULL, or [n,F] values of `dtype` as scratch (not aliasing E or dX).  The rows are
 *           formed inside the products when K and F are whole 16-byte pieces, D is too,
 *           F <= 256, H <= 16 (bf16: H <= 8) and the pointers are 16-byte aligned; for any
 *           other shape they are written to `rows` first (same values), and without
 *           `rows` such a shape returns SAR_ERR_UNSUPPORTED.  With `rows` given they are
 *           always written there, so a caller who wants E_p as well passes it.
 * X [n,K], W [K,F], dW, dX, work as in sar_linear_bwd (F = H*D). */
int sar_linear_bwd_rows(const void* X, const void* E, const int32_t* E_rank, int64_t n_E, const float* ds,
                        const float* a_r, int H, int D, const float* W, float* dW, void* dX, int dtype,
                        int64_t n, int K, void* rows, void* work, size_t work_bytes, void* stream);

int sar_linear_workspace_bytes(int64_t n, int K, int F, size_t* bytes);

#ifdef __cplusplus
}
#endif
#endif /* SAR_MI355X_H */
