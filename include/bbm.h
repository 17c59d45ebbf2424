/*
 * bbm.h -- C ABI of libbbm: Binary Block Masking flash attention (forward and backward) for AMD MI355X (gfx950).
 *
 * The library implements the two stages of the paper "Efficiently Dispatching Flash Attention For Partially
 * Filled Attention Masks" (Sec. 4, Method): (1) reduce an N x N binary attention mask to a block matrix at
 * the attention kernel's Br x Bc tile size, plus the run index of the "Dense" variant and a compact per-row
 * list of non-zero blocks; (2) a fused attention forward that visits only non-zero key/value tiles and
 * applies the element mask only on partially filled tiles.
 *
 * Conventions common to every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller (the only host pointer is the `bbm_index*`
 *     struct itself).  The library never allocates, frees or retains caller memory and never synchronises:
 *     all work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Return value: BBM_OK (0) or a negative error code; bbm_last_error() gives a thread-local message.
 *     Arguments are validated on the host BEFORE any GPU call, so invalid arguments never reach a kernel.
 *     On error the outputs are unspecified.
 *   - Mb is the number of mask planes: 1 (one mask shared by the whole batch) or B (one per batch entry).
 *     A mask is always shared by all heads (paper Sec. 1, insight (2); Sec. 4).
 *   - nbr = ceil(N / Br), nbc = ceil(N / Bc).  The mask is treated as zero-padded to nbr*Br x nbc*Bc (the
 *     paper assumes N divisible by the block size); a block that contains padding is never "full".
 */
#ifndef BBM_H
#define BBM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BBM_OK 0
#define BBM_EINVAL (-1)       /* NULL / misaligned pointer, non-positive size, inconsistent arguments */
#define BBM_EUNSUPPORTED (-2) /* no kernel instance for this (d, Br, Bc) or block size               */
#define BBM_EWORKSPACE (-3)   /* workspace smaller than bbm_attn_fwd_workspace_bytes(), or a problem beyond the static
                                 scratch of bbm_attn_fwd_static                                       */
#define BBM_EHIP (-4)         /* the HIP runtime reported a launch failure                            */

/* Block classes written by bbm_build_block_mask (paper Appendix A: the block sum decides both outputs). */
#define BBM_BLOCK_EMPTY 0   /* every element of the block is zero        */
#define BBM_BLOCK_PARTIAL 1 /* some, not all, elements are non-zero      */
#define BBM_BLOCK_FULL 2    /* all Br*Bc elements are non-zero           */

/* Tile schedules of bbm_attn_fwd. */
#define BBM_MODE_BITMAP 0         /* paper Sec. 4 "Binary Block Masking": visit block (i,j) iff BinBlkMat[i][j]; element
                                     mask applied on every visited block                                               */
#define BBM_MODE_RUNS 1           /* paper Sec. 4 "Dense Binary Block Masking": scan [nz_lo, nz_hi), visit iff BinBlkMat,
                                     skip the element mask inside [offset, offset + total_ones)                        */
#define BBM_MODE_LIST 2           /* walk the compact per-row list of non-zero blocks; element mask skipped on blocks
                                     flagged full; rows the split schedule cut are computed part by part by extra
                                     work-groups and merged                                                            */
/* Small launches, all three schedules above: at most 256 work-groups (B*H*nbr) over long rows leave compute units idle
 * or with a single work-group, so EVERY block row is computed in min(8, 512 / (B*H*nbr), nbc / t) equal parts (of its
 * list, resp. of the block columns) by as many work-groups and merged in part order; t = 32 block columns below 128
 * work-groups, 64 from there on; fewer than 2 parts means none.  This needs the workspace; BITMAP and RUNS, which
 * otherwise need none, run one work-group per block row when none is given. */
#define BBM_MODE_DENSE_BASELINE 3 /* paper Sec. 3 "naive masking": visit every block, apply the element mask everywhere */
#define BBM_MODE_AUTO 4           /* LIST if the index carries list and schedule, else RUNS, else BITMAP               */

/* Device pointers produced by the build functions, gathered for bbm_attn_fwd.  The struct lives in host
 * memory; unused members may be NULL (which ones are needed depends on `mode`, see bbm_attn_fwd). */
typedef struct bbm_index {
  int32_t Br, Bc;             /* tile size the index was built for                                   */
  int64_t Mb, nbr, nbc;       /* planes, block rows, block columns                                   */
  int64_t Nq, Nk;             /* query rows and key columns of the mask the index was built from (the packed mask's
                                 row stride is Nq, so a tensor of another length must be refused even where it gives
                                 the same block counts)                                                   */
  const uint8_t* blk_class;   /* [Mb, nbr, nbc] BBM_BLOCK_*                                          */
  const uint8_t* bin_blk_mat; /* [Mb, nbr, nbc] 0/1, the paper's BinBlkMat                           */
  const int32_t* offset;      /* [Mb, nbr] first block of the longest run of full blocks             */
  const int32_t* total_ones;  /* [Mb, nbr] length of that run                                        */
  const int32_t* nz_lo;       /* [Mb, nbr] first non-zero block                                      */
  const int32_t* nz_hi;       /* [Mb, nbr] one past the last non-zero block                          */
  const int32_t* nz_cnt;      /* [Mb, nbr] number of non-zero blocks                                 */
  const int32_t* row_ptr;     /* [Mb, nbr + 1] list offsets within a plane, row_ptr[m][0] = 0        */
  const uint32_t* col_idx;    /* [Mb * nbr * nbc]; plane m starts at m*nbr*nbc; bit 31 = block full  */
  const int32_t* sched;       /* bbm_sched_bytes(Mb, nbr) bytes: tile schedule of LIST mode           */
  const int32_t* col_ptr;     /* [Mb, nbc + 1] column-list offsets within a plane (backward pass)    */
  const uint32_t* row_idx;    /* [Mb * nbr * nbc]; plane m starts at m*nbr*nbc; bit 31 = block full  */
  const int32_t* col_sched;   /* bbm_col_sched_bytes(Mb, nbc) bytes: split schedule of the column walk */
} bbm_index;

/* Thread-local description of the last error returned on this thread ("" if none). */
const char* bbm_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int bbm_version(void);

/*
 * Stage 1a -- block reduction (paper Sec. 4 "Binary Block Masking": entry (i,j) of BinBlkMat is 1 iff any
 * element of mask block (i,j) is non-zero; Appendix A, block-based summation kernel).
 *
 *   mask             device, uint8 [Mb][N][row_stride_bytes]; element (m, r, c) at
 *                    mask + (m*N + r)*row_stride_bytes + c; any non-zero byte means "query r may attend key c".
 *                    row_stride_bytes >= N.  The fast path needs mask and row_stride_bytes 16-byte aligned;
 *                    other alignments take a slower byte-wise path with identical results.
 *   Br, Bc           block size; 1 <= Br <= 256; Bc in {16, 32, 64, 128, 256}.
 *   blk_class        device out, uint8 [Mb][nbr][nbc], BBM_BLOCK_* (required).
 *   bin_blk_mat      device out, uint8 [Mb][nbr][nbc], 0/1; may be NULL.
 *   packed_mask      device out, uint64 [Mb][W][N] with W = ceil(N/64), word-column major: bit t of word
 *                    (m, w, r) is (mask[m][r][64*w + t] != 0), bits for columns >= N are zero; may be NULL.
 *                    Must be 8-byte aligned.  This is the form in which bbm_attn_fwd reads the element mask.
 *                    Words are written per slab of one block row x 64 columns (rows [i*Br, (i+1)*Br) of word column
 *                    w), and ONLY for slabs that hold a set bit: an all-zero slab keeps whatever the buffer held.
 *                    With Bc = 64 a slab is a block and the unwritten ones are exactly the BBM_BLOCK_EMPTY blocks,
 *                    which no schedule visits (BBM_MODE_DENSE_BASELINE takes their zeros from the class bytes); on a
 *                    sparse mask that is most of the output, and the writes cost more than their share of the bytes.
 * Errors: BBM_EINVAL (NULL mask/blk_class, Mb/N < 1, stride < N, misaligned packed_mask),
 *         BBM_EUNSUPPORTED (block size outside the ranges above), BBM_EHIP.
 */
int bbm_build_block_mask(const uint8_t* mask, int64_t Mb, int64_t N, int64_t row_stride_bytes, int Br, int Bc,
                         uint8_t* blk_class, uint8_t* bin_blk_mat, uint64_t* packed_mask, void* stream);

/*
 * The same reduction for a rectangular mask: Nq query rows x Nk key columns (a block of new tokens attending a longer
 * key/value cache, e.g. a candidate tree verified against its prefix, paper Sec. 5).  mask is uint8
 * [Mb][Nq][row_stride_bytes] with row_stride_bytes >= Nk; nbr = ceil(Nq/Br), nbc = ceil(Nk/Bc); packed_mask is
 * uint64 [Mb][ceil(Nk/64)][Nq].  bbm_build_block_mask(.., N, ..) is this call with Nq = Nk = N; same errors.  The index
 * builders below take nbr and nbc and need no rectangular form.
 */
int bbm_build_block_mask_rect(const uint8_t* mask, int64_t Mb, int64_t Nq, int64_t Nk, int64_t row_stride_bytes, int Br,
                              int Bc, uint8_t* blk_class, uint8_t* bin_blk_mat, uint64_t* packed_mask, void* stream);

/*
 * Stage 1b -- contiguous-run index (paper Sec. 4 "Dense Binary Block Masking": per block row, total_ones =
 * number of consecutive blocks filled with ones, offset = position of the first such block).
 * Reading fixed here: "filled with ones" = BBM_BLOCK_FULL; if a row has several runs the longest is kept,
 * the leftmost on ties; no full block gives (offset, total_ones) = (0, 0).  In addition the span of
 * non-zero blocks is reported: nz_lo = first non-zero block, nz_hi = one past the last, nz_cnt = how many
 * ((0,0,0) for an empty row); the row's non-zero blocks are contiguous iff nz_cnt == nz_hi - nz_lo.
 *
 *   blk_class        device in, uint8 [Mb][nbr][nbc] from bbm_build_block_mask.
 *   offset, total_ones, nz_lo, nz_hi, nz_cnt   device out, int32 [Mb][nbr] each (all required).
 * Errors: BBM_EINVAL (NULL pointer, non-positive size), BBM_EHIP.
 */
int bbm_build_runs(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, int32_t* offset,
                   int32_t* total_ones, int32_t* nz_lo, int32_t* nz_hi, int32_t* nz_cnt, void* stream);

/*
 * Stage 1c -- compact per-row list of non-zero blocks, for very sparse masks (the abstract's second
 * refinement; the list layout is this library's: CSR over block rows).
 *
 *   blk_class        device in, uint8 [Mb][nbr][nbc].
 *   row_ptr          device out, int32 [Mb][nbr + 1]; row_ptr[m][0] = 0, row_ptr[m][i+1] - row_ptr[m][i] =
 *                    number of non-zero blocks of block row i.
 *   col_idx          device out, uint32, capacity Mb*nbr*nbc entries; the list of plane m starts at entry
 *                    m*nbr*nbc; block columns ascending within a row; bit 31 set iff the block is full.
 *                    Entries past row_ptr[m][nbr] are left untouched.
 *   sched            device out, bbm_sched_bytes(Mb, nbr) bytes, 32-byte aligned; may be NULL.  The split schedule
 *                    that LIST mode of bbm_attn_fwd uses to keep one very long block row (a row of global tokens,
 *                    say) from becoming the whole kernel's critical path: rows with more than
 *                    T = max(32, 2 * mean entries per non-empty row) list entries are cut into ceil(n/T) near-equal
 *                    parts.  int32 layout: [0] parts, [1] T, [2] cut rows, [3..7] 0, then 8 ints per part ordered by
 *                    (row, part): plane*nbr + block row, first entry (position in the plane's list), entries, part,
 *                    parts of the row, number of the row's first part, index of the row among the cut rows, the list
 *                    entry at the part's first position.
 *                    The last 4*Mb*nbr ints are one 4-int record per (plane, rank), in the order in which LIST mode
 *                    starts the block rows of a plane: groups of 4 consecutive block rows if T = 32, i.e. while rows
 *                    are short (neighbours share most of their key/value tiles, so they should run at the same time),
 *                    else single rows (with long rows the plain longest-first order balances the tail better); the
 *                    groups by the list length of their longest row, longest first (ties: the group of higher rows
 *                    first), the rows of a group by list length, longest first (ties: higher row first); planes with
 *                    more than 4096 block rows: simply last row first.
 *                    A record holds the block row, the position of its first entry in the plane's list, its number of
 *                    entries and its first list entry (-1 if it has none), i.e. all a work-group needs to start
 *                    fetching.
 *                    It depends only on the mask, so it is shared by heads, layers and calls like the rest of the
 *                    index.
 * Requires nbr*nbc < 2^31 and Mb*nbr < 2^24.  Errors: BBM_EINVAL, BBM_EHIP.
 */
int bbm_build_sparse_index(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, int32_t* row_ptr,
                           uint32_t* col_idx, int32_t* sched, void* stream);

/*
 * Stages 1b and 1c in one call: exactly the outputs of bbm_build_runs followed by bbm_build_sparse_index (same
 * arguments, same requirements, same errors), none of the output pointers except sched may be NULL.  Class matrices
 * of at most 256 (block row, 64-column chunk) pairs -- 4 planes of a 4096 x 4096 mask in 128 x 64 tiles, say -- are
 * served by a single kernel launch, which at that size is most of the cost.
 */
int bbm_build_index(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, int32_t* offset, int32_t* total_ones,
                    int32_t* nz_lo, int32_t* nz_hi, int32_t* nz_cnt, int32_t* row_ptr, uint32_t* col_idx, int32_t* sched,
                    void* stream);

/* Bytes of the tile schedule bbm_build_sparse_index writes for Mb planes of nbr block rows (0 for sizes < 1). */
size_t bbm_sched_bytes(int64_t Mb, int64_t nbr);

/*
 * Bytes of device workspace bbm_attn_fwd needs for this problem (0 if none).  Negative sizes return 0.  LIST (and AUTO)
 * must be given it; for BITMAP and RUNS it is what a small launch (see the modes) needs to be computed in parts, and
 * optional.
 * Layout: (8 + B*H*ceil(N/Br)) int32 queue counters, rounded up to 256 bytes -- the only part that has to be zero --
 * then room for partial results: (d/2 + 2) * 2*Br floats per record, one record per (cut part, batch, head) resp.
 * per (block row, part, batch, head) of a small launch.  The room for cut rows stops at 32 MiB; a schedule whose parts
 * need more records than the workspace holds is not followed (those rows are computed whole by one work-group).
 */
size_t bbm_attn_fwd_workspace_bytes(int64_t B, int64_t H, int64_t N, int d, int Br, int Bc, int mode);

/*
 * Stage 2 -- fused masked attention forward (paper Sec. 3 "Standard Attention"/"Flash Attention", Sec. 4):
 * for every batch b, head h and query i with allowed key set A_i = { j : mask[m(b)][i][j] != 0 },
 *     O[b,h,i,:] = sum_{j in A_i} softmax_{j in A_i}(softmax_scale * <q_i, k_j>) * v_j
 *     lse[b,h,i] = log sum_{j in A_i} exp(softmax_scale * <q_i, k_j>)
 * computed tile by tile with an online softmax; only blocks the index marks non-zero are visited and the
 * element mask is applied only where the schedule says a block may be partial.  A query with A_i empty
 * gets O = 0 and lse = -inf.  m(b) = b if Mb == B, else 0.
 *
 *   q, k, v          device in, bf16 [B][H][N][d] contiguous, 16-byte aligned.
 *   o                device out, bf16 [B][H][N][d] contiguous (round-to-nearest-even), 16-byte aligned.
 *   lse              device out, fp32 [B][H][N] natural-log-sum-exp; may be NULL.
 *   d                head dimension: 64 or 128.
 *   softmax_scale    finite and > 0 (1/sqrt(d) is the usual choice; the paper does not name one).
 *   packed_mask      device in, uint64 [Mb][ceil(N/64)][N] from bbm_build_block_mask.
 *   idx              host pointer; idx->Bc must be 64 and idx->Br one of 64, 128, 256; idx->Mb == Mb;
 *                    idx->Nq = idx->Nk = N and idx->nbr/nbc = ceil(N/Br), ceil(N/Bc).  Members needed per mode:
 *                    BITMAP: bin_blk_mat;  RUNS: bin_blk_mat, offset, total_ones, nz_lo, nz_hi;
 *                    LIST: row_ptr, col_idx, sched;  DENSE_BASELINE: bin_blk_mat or blk_class (an empty block has no packed words).
 *   mode             BBM_MODE_*.
 *   workspace        device scratch of at least bbm_attn_fwd_workspace_bytes(...) bytes, 16-byte aligned (may be NULL
 *                    if 0).  LIST mode keeps its queue counters and the partial results of cut block rows there.
 *                    The workspace's counters (see bbm_attn_fwd_workspace_bytes; zero-filling all of it is fine too)
 *                    must be ZERO-FILLED ONCE after it is allocated; every call puts back the zeros it disturbed, so
 *                    the same workspace can serve any number of later calls of the same (B, H, N, d, Br) without being
 *                    cleared again.  Before a call of another shape clear the counters again: one shape's partial
 *                    results may lie where another shape's counters do.  Two calls that overlap in time (different streams) must not
 *                    share a workspace.
 * Arithmetic: QK^T and PV on bf16 MFMA with fp32 accumulation; softmax statistics in fp32; P rounded to bf16 before PV
 * and the row sum adds the rounded P.  For softmax_scale <= 1/sqrt(d) (the usual choice and anything flatter) Q is
 * multiplied by softmax_scale*log2(e) and rounded to bf16 once, so the first product yields base-2 exponents directly
 * (a score moves by at most 2^-9 * softmax_scale * sum_c |q_c k_c|).  For sharper scales that rounding would grow with
 * the scale, so only the power-of-two part of softmax_scale*log2(e) goes into Q (exact in bf16) and the rest multiplies
 * the first product's fp32 result: the same accuracy at every scale, for one more multiplication per score.  Deterministic: the same inputs give bit-identical outputs (in LIST mode the parts of a cut row
 * are taken from a queue in whatever order work-groups become free, but each part's arithmetic and the order in
 * which the parts are merged are fixed).
 * Errors: BBM_EINVAL, BBM_EUNSUPPORTED (d / Br / Bc without a kernel instance), BBM_EWORKSPACE, BBM_EHIP.
 */
int bbm_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B, int64_t H, int64_t N,
                 int d, float softmax_scale, int64_t Mb, const uint64_t* packed_mask, const bbm_index* idx, int mode,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * bbm_attn_fwd for Nq queries against Nk keys per (batch, head): q and o are [B][H][Nq][d], k and v [B][H][Nk][d], lse
 * [B][H][Nq], packed_mask [Mb][ceil(Nk/64)][Nq] from bbm_build_block_mask_rect, idx->nbr = ceil(Nq/Br), idx->nbc =
 * ceil(Nk/Bc), idx->Nq = Nq, idx->Nk = Nk.  Everything else as bbm_attn_fwd, which is this call with Nq = Nk = N; the workspace size is
 * bbm_attn_fwd_workspace_bytes(B, H, Nq, ...).
 */
int bbm_attn_fwd_rect(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B, int64_t H, int64_t Nq,
                      int64_t Nk, int d, float softmax_scale, int64_t Mb, const uint64_t* packed_mask,
                      const bbm_index* idx, int mode, void* workspace, size_t workspace_bytes, void* stream);

/*
 * bbm_attn_fwd_rect for callers that cannot allocate device memory and have no workspace to hand over: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus the workspace),
 * same kernels, same results; the queue counters and partial results of LIST mode live in a 32 MiB array that is part
 * of the library's device code (every GPU the library runs on holds its own copy until the process ends).  The call
 * allocates and frees nothing.
 *   - Limit: the counters, 4 * (8 + B*H*ceil(Nq/Br)) bytes, plus one partial record must fit in the 32 MiB, else
 *     BBM_EWORKSPACE (use bbm_attn_fwd_rect with a workspace).  What fits beyond that decides how the work is cut: a
 *     small launch computes its block rows in as many parts as find room, and a schedule whose cut parts do not all
 *     find room is not followed (same results up to the rounding order of the merge; slower on such masks).
 *   - The call clears the counters it uses with a fill kernel on `stream` before the attention kernel; the array
 *     otherwise keeps the last call's contents.
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different streams, or
 *     different host threads without ordering) race.  Calls on different GPUs do not interact.
 *   - The current device must be the one `stream` and the data pointers belong to.  The first call on a device looks up
 *     the array's address (which loads the library's device code there): make that call outside graph capture.
 * Errors: as bbm_attn_fwd_rect, BBM_EWORKSPACE as above, BBM_EUNSUPPORTED for device ordinals of 64 and above.
 */
int bbm_attn_fwd_static(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B, int64_t H, int64_t Nq,
                        int64_t Nk, int d, float softmax_scale, int64_t Mb, const uint64_t* packed_mask,
                        const bbm_index* idx, int mode, void* stream);

/*
 * Per-column list of non-zero blocks, the transpose of the list of bbm_build_sparse_index: what the dK/dV step of
 * the backward pass walks (a block of keys visits the query blocks that may attend it; paper Sec. 4: only non-zero
 * blocks are processed, in the backward pass as in the forward).
 *
 *   blk_class        device in, uint8 [Mb][nbr][nbc].
 *   col_ptr          device out, int32 [Mb][nbc + 1]; col_ptr[m][0] = 0, col_ptr[m][j+1] - col_ptr[m][j] = number of
 *                    non-zero blocks of block column j.
 *   row_idx          device out, uint32, capacity Mb*nbr*nbc entries; the list of plane m starts at entry m*nbr*nbc;
 *                    block rows ascending within a column; bit 31 set iff the block is full.  Entries past
 *                    col_ptr[m][nbc] are left untouched.
 *   col_sched        device out, bbm_col_sched_bytes(Mb, nbc) bytes, 32-byte aligned; may be NULL.  The split schedule
 *                    that keeps one very long block column (a block of global keys, say) from becoming the critical
 *                    path of the dK/dV step: columns with more than T = max(16, 2 * mean entries per non-empty
 *                    column) list entries are cut into ceil(n/T) near-equal parts.  int32 layout as the part table of
 *                    bbm_build_sparse_index's schedule: [0] parts, [1] T, [2] cut columns, [3..7] 0, then 8 ints per
 *                    part ordered by (column, part): plane*nbc + block column, first entry (position in the plane's
 *                    list), entries, part, parts of the column, number of the column's first part, index of the column
 *                    among the cut columns, the list entry at the part's first position.  The last 4*Mb*nbc ints are one
 *                    4-int record per (plane, rank) in the order in which the dK/dV step starts the block columns of a
 *                    plane: by list length, longest first (ties: the higher column first; planes with more than 4096
 *                    block columns: simply last column first); a record holds the block column, the position of its
 *                    first entry in the plane's list, its number of entries and its first list entry (-1 if none).
 * Requires nbr*nbc < 2^31, and Mb*nbc < 2^24 if col_sched is given.  Errors: BBM_EINVAL, BBM_EHIP.
 */
int bbm_build_col_index(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, int32_t* col_ptr,
                        uint32_t* row_idx, int32_t* col_sched, void* stream);

/* Bytes of the column schedule bbm_build_col_index writes for Mb planes of nbc block columns (0 for sizes < 1). */
size_t bbm_col_sched_bytes(int64_t Mb, int64_t nbc);

/* Bytes of device workspace bbm_attn_bwd needs for this problem (0 for sizes < 1 or a (d, Br) without a kernel). */
size_t bbm_attn_bwd_workspace_bytes(int64_t B, int64_t H, int64_t N, int d, int Br);

/*
 * Backward pass of bbm_attn_fwd (paper Sec. 3 "Flash Attention": the attention matrix is recomputed block by block
 * from the stored log-sum-exp; Sec. 4: only non-zero blocks are visited, the element mask is applied on partial ones
 * only; Sec. 5 and the appendix on forward and backward runtimes time both passes).  For an upstream gradient dO and
 * p_ij = exp(softmax_scale * <q_i, k_j> - lse_i) for j in A_i, 0 elsewhere:
 *     dV_j = sum_i p_ij dO_i,   D_i = <dO_i, O_i>,   dS_ij = p_ij (<dO_i, v_j> - D_i),
 *     dQ_i = softmax_scale * sum_j dS_ij k_j,        dK_j = softmax_scale * sum_i dS_ij q_i.
 * A query with A_i empty (lse = -inf) contributes nothing and gets dQ = 0; a key nobody attends gets dK = dV = 0.
 *
 *   q, k, v, o, d_o  device in, bf16 [B][H][N][d] contiguous, 16-byte aligned; o and lse as bbm_attn_fwd returned them.
 *   lse              device in, fp32 [B][H][N] (required).
 *   dq, dk, dv       device out, bf16 [B][H][N][d] contiguous (round-to-nearest-even), 16-byte aligned; every element
 *                    is written.
 *   d, softmax_scale, Mb, packed_mask   as for bbm_attn_fwd (the same values as in the forward call).
 *   idx              host pointer; Br, Bc, Mb, nbr, nbc as for bbm_attn_fwd; needs row_ptr, col_idx (the dQ step walks
 *                    block rows), col_ptr, row_idx (the dK/dV step walks block columns).  If sched resp. col_sched is
 *                    present, block rows resp. columns the schedule cut are computed part by part by the leading
 *                    work-groups and summed in part order (and sched gives the launch order of the block rows).
 *   workspace        device scratch of at least bbm_attn_bwd_workspace_bytes(B, H, N, d, idx->Br) bytes, 16-byte
 *                    aligned; holds the queue counters, D and the log-sum-exp in the form the second kernel consumes,
 *                    and the fp32 partial sums of cut rows and columns (an upper bound: most of it is never touched).
 *                    Like the forward workspace it must be ZERO-FILLED ONCE after it is allocated; every call puts
 *                    back the zeros it disturbed (its two counter arrays come first: 8 + B*H*nbr and 8 + B*H*nbc int32,
 *                    each rounded up to 256 bytes); clear them again before a call of another shape.  Two calls that overlap in time must not share a workspace.
 * Arithmetic: all five products on bf16 MFMA with fp32 accumulation; Q (dQ step) resp. K (dK/dV step) is multiplied by
 * softmax_scale*log2(e) and rounded to bf16 once (for scales sharper than 1/sqrt(d): by its power-of-two part only, the
 * rest being applied in fp32, as in bbm_attn_fwd); P and dS are rounded to bf16 before the products that consume them.
 * Two kernels, no floating-point atomics: the same inputs give bit-identical outputs (parts of a cut row or column are
 * taken from a queue in whatever order work-groups become free, but are summed in part order).
 * Errors: BBM_EINVAL, BBM_EUNSUPPORTED, BBM_EWORKSPACE, BBM_EHIP.
 */
int bbm_attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* d_o, const float* lse, void* dq,
                 void* dk, void* dv, int64_t B, int64_t H, int64_t N, int d, float softmax_scale, int64_t Mb,
                 const uint64_t* packed_mask, const bbm_index* idx, void* workspace, size_t workspace_bytes,
                 void* stream);

/*
 * Reverse Cuthill-McKee reordering of a sparse mask (paper Sec. 4 "Binary Block Masking with Reverse Cuthill-McKee
 * (RCM)": the mask is treated as the adjacency matrix of a graph and reordered so that fewer blocks are non-zero).
 * The published algorithm with every choice fixed: the neighbours of node i are the non-zero entries of mask row i
 * (the mask is read row-wise; the method assumes a symmetric mask), its degree their number; each connected component
 * starts at its unvisited node of minimum degree (ties: smallest index); breadth-first, each level ordered by (position
 * of the node's earliest parent in the ordering, degree, index); the ordering is reversed at the end.
 *
 *   mask             device in, uint8 [N][row_stride_bytes], one plane, row_stride_bytes >= N (16-byte aligned pointer
 *                    and stride take the fast path).
 *   perm             device out, int32 [N]: perm[k] = old index of the node placed at position k; the reordered mask is
 *                    mask[perm][:, perm] (bbm_permute_mask), reordered Q/K/V rows are row perm[k] at position k
 *                    (bbm_gather_rows), and O comes back with the inverse (bbm_gather_rows with inverse = 1).
 *   workspace        device scratch of at least bbm_rcm_workspace_bytes(N) bytes (N*ceil(N/64)*8 for the packed rows
 *                    plus about 26*N), 16-byte aligned; needs no initialisation.
 * N <= 65536.  No host round trip: a fixed number of rounds (one breadth-first level or one component start each) use
 * the whole GPU, a one-work-group finisher walks whatever is left; so time grows with the number of levels and of
 * connected components beyond 48 (each costs one work-group a scan over the N nodes).
 * Errors: BBM_EINVAL, BBM_EUNSUPPORTED (N > 65536), BBM_EWORKSPACE, BBM_EHIP.
 */
size_t bbm_rcm_workspace_bytes(int64_t N);
int bbm_rcm_order(const uint8_t* mask, int64_t N, int64_t row_stride_bytes, int32_t* perm, void* workspace,
                  size_t workspace_bytes, void* stream);

/*
 * out[m][i][j] = mask[m][perm[i]][perm[j]] for Mb planes (uint8, out contiguous [Mb][N][N], out != mask).  N <= 65536.
 * Entries of perm outside [0, N) are clamped.  Errors: BBM_EINVAL, BBM_EUNSUPPORTED, BBM_EHIP.
 */
int bbm_permute_mask(const uint8_t* mask, int64_t Mb, int64_t N, int64_t row_stride_bytes, const int32_t* perm,
                     uint8_t* out, void* stream);

/*
 * Rows of a bf16 tensor [BH][N][d] (d a multiple of 8, 16-byte aligned, out != in): inverse = 0 gathers,
 * out[bh][k] = in[bh][perm[k]] (Q, K, V into the reordered problem); inverse = 1 scatters, out[bh][perm[k]] = in[bh][k]
 * (O back to the original order).  Errors: BBM_EINVAL, BBM_EUNSUPPORTED, BBM_EHIP.
 */
int bbm_gather_rows(const void* in, const int32_t* perm, void* out, int64_t BH, int64_t N, int d, int inverse,
                    void* stream);

/* ---- Hardware-ceiling probe (measurement aid, no part of the method) -------------------------------------------- */

/*
 * Launches one kernel that issues only `v_mfma_f32_32x32x16_bf16` instructions: 256 work-groups of 4 waves (one wave
 * per SIMD of a 256-CU chip), each wave `iters` times a chain of 16 instructions over four accumulators, operands held
 * in registers.  normal_operands = 0: every operand element is one small constant; != 0: seeded, nearly normal values
 * of unit variance, different in every lane and fragment (the arithmetic units draw more power on such operands, and
 * the chip lowers its clock accordingly, so this is the matrix rate a kernel fed with real data can be set against).
 * The caller times the launch (events on `stream`); bbm_probe_mfma_bf16_flop(iters) is the flop count of one launch.
 *   sink             device out, float [65536]: one value per thread, written so that the work cannot be dropped.
 *   iters            1 .. 2^24 (100000 runs for about 25 ms).
 * Errors: BBM_EINVAL, BBM_EHIP.
 */
int bbm_probe_mfma_bf16(int normal_operands, int64_t iters, float* sink, void* stream);
double bbm_probe_mfma_bf16_flop(int64_t iters);

#ifdef __cplusplus
}
#endif
#endif /* BBM_H */
