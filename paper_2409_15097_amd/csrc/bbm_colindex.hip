// Per-column list of non-zero blocks: the transpose of the block list, walked by the dK/dV step of the backward pass
// (one work-group owns a block of keys and visits the query blocks that may attend it; paper Sec. 4: only non-zero
// blocks are processed).
#include "bbm_internal.h"

namespace {

constexpr int kColThreads = 1024;

// One work-group per mask plane; a thread owns one block column of the current chunk of kColThreads columns, counts
// its non-zero blocks, the work-group scans the counts, and the thread then writes its column's entries.
__global__ __launch_bounds__(kColThreads) void col_index_kernel(const uint8_t* __restrict__ cls, int nbr, int nbc,
                                                                int32_t* __restrict__ col_ptr, uint32_t* __restrict__ row_idx) {
  __shared__ int wave_tot[kColThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t m = blockIdx.x;
  const uint8_t* __restrict__ plane = cls + m * nbr * nbc;
  uint32_t* __restrict__ out = row_idx + m * nbr * nbc;
  int32_t* __restrict__ cp = col_ptr + m * (nbc + 1);
  int base = 0;  // entries of all earlier chunks (uniform)
  for (int j0 = 0; j0 < nbc; j0 += kColThreads) {
    const int j = j0 + tid;
    const bool ok = j < nbc;
    int cnt = 0;
    if (ok) {
#pragma unroll 8
      for (int i = 0; i < nbr; ++i) cnt += plane[(int64_t)i * nbc + j] != 0 ? 1 : 0;
    }
    // exclusive scan over the work-group: inclusive scan inside the wave, then the totals of the earlier waves
    int incl = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d);
      if (lane >= d) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int before = 0, chunk_total = 0;
    for (int w = 0; w < kColThreads / 64; ++w) {
      const int t = wave_tot[w];
      if (w < wave) before += t;
      chunk_total += t;
    }
    __syncthreads();  // wave_tot is rewritten by the next chunk
    int pos = base + before + incl - cnt;
    if (ok) {
      cp[j] = pos;
      for (int i = 0; i < nbr; ++i) {
        const uint8_t c = plane[(int64_t)i * nbc + j];
        if (c != 0) out[pos++] = (uint32_t)i | (c == BBM_BLOCK_FULL ? 0x80000000u : 0u);
      }
    }
    base += chunk_total;
  }
  if (tid == 0) cp[nbc] = base;
}

}  // namespace

extern "C" __attribute__((visibility("default"))) int bbm_build_col_index(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc,
                                                                         int32_t* col_ptr, uint32_t* row_idx, void* stream) {
  using namespace bbm;
  clear_error();
  if (!blk_class || !col_ptr || !row_idx) return fail(BBM_EINVAL, "bbm_build_col_index: blk_class, col_ptr, row_idx must not be NULL");
  if (Mb < 1 || nbr < 1 || nbc < 1)
    return fail(BBM_EINVAL, "bbm_build_col_index: Mb=%lld, nbr=%lld, nbc=%lld must be >= 1", (long long)Mb, (long long)nbr, (long long)nbc);
  if (!aligned(col_ptr, 4) || !aligned(row_idx, 4)) return fail(BBM_EINVAL, "bbm_build_col_index: col_ptr, row_idx must be 4-byte aligned");
  if (nbr * nbc >= (1ll << 31) || Mb >= (1ll << 31)) return fail(BBM_EINVAL, "bbm_build_col_index: nbr*nbc and Mb must be below 2^31");
  col_index_kernel<<<(unsigned)Mb, kColThreads, 0, static_cast<hipStream_t>(stream)>>>(blk_class, (int)nbr, (int)nbc, col_ptr, row_idx);
  return launch_status("bbm_build_col_index");
}
