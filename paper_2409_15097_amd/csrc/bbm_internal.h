// Internal helpers shared by the translation units of libbbm (host side only; no kernels live here).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "bbm.h"

namespace bbm {

// Records a thread-local message and returns `code` so call sites can `return fail(...)`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Checks the launch status of the kernel just enqueued.
inline int launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(BBM_EHIP, "%s: %s", what, hipGetErrorString(e));
  return BBM_OK;
}

// Layout of the split schedule that bbm_build_sparse_index writes and bbm_attn_fwd (LIST mode) reads; int32 units.
//   [kSchedNParts]           number of parts (0 if no block row was cut)
//   [kSchedSplitT]           split threshold T: block rows with more than T list entries are cut into parts
//   [kSchedNCutRows]         number of block rows that were cut
//   [kSchedPartBase + 8*q]   part q (ordered by row, then part): row (= plane*nbr + block row), first entry in the
//                            plane's list, entries, part index, parts of the row, q of the row's first part, index
//                            of the row among the cut rows, list entry at the part's first position
//   [order_base + 4*(m*nbr + k)]  record of the k-th block row of plane m in launch order: block row, position of
//                            its first entry in the plane's list, entries, first list entry (-1 if none);
//                            order_base = kSchedPartBase + 8*Mb*nbr.  Launch order: groups of kSchedGroupRows
//                            consecutive rows if T is at its floor, else single rows; the group holding the longest row
//                            first (ties: higher rows first), inside a group the longest row first (ties: higher row first); planes with more
//                            than kSchedMaxSortRows block rows are simply listed from the last row to the first
constexpr int kSchedNParts = 0, kSchedSplitT = 1, kSchedNCutRows = 2;
constexpr int kSchedPartBase = 8;
constexpr int kSchedPartInts = 8;
constexpr int kSchedMinSplit = 32;
constexpr int kSchedMaxSortRows = 4096;
constexpr int kSchedRowInts = 4;
constexpr int kSchedGroupRows = 4;
// Column schedule of the backward pass (bbm_build_col_index writes it, bbm_attn_bwd reads it): the same header and
// 8-int part records with block columns in place of block rows, launch-order records of single columns (longest
// first; ties: higher column first) after the Mb*nbc part slots, and a lower floor of the
// split threshold (a column entry stands for Br/64 sub-tiles of twice the work of a forward tile).
constexpr int kColSchedMinSplit = 16;
__host__ __device__ inline int64_t sched_order_base(int64_t Mb, int64_t nbr) { return kSchedPartBase + kSchedPartInts * Mb * nbr; }
__host__ __device__ inline int64_t sched_ints(int64_t Mb, int64_t nbr) { return sched_order_base(Mb, nbr) + kSchedRowInts * Mb * nbr; }

// Launch order of the attention kernels: how many (batch, head) planes have their block rows (columns) interleaved
// inside one XCD's contiguous share of the launch.  Interleaving lets the long rows of several planes start first
// (packed short sequences: 20-35 % faster with 8 planes than with 1), but the work-groups of one XCD then stream the
// tensors of all those planes through its 4 MiB L2: with heads of 4 MiB (N = 8192, d = 128, dense) 8 planes made
// 41 % of the dK/dV kernel's L2 requests miss against 4 % with one plane, and cost 4-5 % of the run time.  So large
// heads are not interleaved.  `streamed_bytes` is what one plane's work-groups read over and over (K and V, or Q
// and dO, of one head).
constexpr int64_t kInterleaveMaxHeadBytes = 2 << 20;
inline int32_t interleaved_planes(int64_t planes, int64_t streamed_bytes) {
  if (streamed_bytes >= kInterleaveMaxHeadBytes) return 1;
  const int64_t g = planes / 8;
  return (int32_t)(g < 1 ? 1 : g > 8 ? 8 : g);
}

}  // namespace bbm
