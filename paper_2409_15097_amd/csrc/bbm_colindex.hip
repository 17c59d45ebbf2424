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

// The same list in three small launches for larger class matrices (a plane of more than kColOneKernelRows block rows):
// one WAVE per block column, its lanes over 64 block rows at a time (count; scan over the columns of a plane; fill).
constexpr int kColOneKernelRows = 64;
constexpr int kColWaves = 4;

__global__ __launch_bounds__(kColWaves * 64) void col_count_kernel(const uint8_t* __restrict__ cls, int64_t Mb, int nbr, int nbc,
                                                                   int32_t* __restrict__ col_ptr) {
  const int lane = threadIdx.x & 63;
  const int64_t col = (int64_t)blockIdx.x * kColWaves + (threadIdx.x >> 6);
  if (col >= Mb * nbc) return;
  const int64_t m = col / nbc, j = col - m * nbc;
  const uint8_t* __restrict__ c = cls + m * nbr * nbc + j;
  int cnt = 0;
  for (int base = 0; base < nbr; base += 64) {
    const uint8_t v = (base + lane < nbr) ? c[(int64_t)(base + lane) * nbc] : (uint8_t)0;
    cnt += __popcll(__ballot(v != BBM_BLOCK_EMPTY));
  }
  if (lane == 0) col_ptr[m * (nbc + 1) + j + 1] = cnt;
}

// In-place inclusive scan of col_ptr[m][1..nbc], one wave per plane.
__global__ __launch_bounds__(64) void col_scan_kernel(int nbc, int32_t* __restrict__ col_ptr) {
  const int lane = threadIdx.x;
  int32_t* p = col_ptr + (int64_t)blockIdx.x * (nbc + 1);
  int carry = 0;
  for (int base = 0; base < nbc; base += 64) {
    int x = (base + lane < nbc) ? p[base + lane + 1] : 0;
    for (int s = 1; s < 64; s <<= 1) {
      const int y = __shfl_up(x, s);
      if (lane >= s) x += y;
    }
    x += carry;
    if (base + lane < nbc) p[base + lane + 1] = x;
    carry = __shfl(x, 63);
  }
  if (lane == 0) p[0] = 0;
}

__global__ __launch_bounds__(kColWaves * 64) void col_fill_kernel(const uint8_t* __restrict__ cls, int64_t Mb, int nbr, int nbc,
                                                                  const int32_t* __restrict__ col_ptr, uint32_t* __restrict__ row_idx) {
  const int lane = threadIdx.x & 63;
  const int64_t col = (int64_t)blockIdx.x * kColWaves + (threadIdx.x >> 6);
  if (col >= Mb * nbc) return;
  const int64_t m = col / nbc, j = col - m * nbc;
  const uint8_t* __restrict__ c = cls + m * nbr * nbc + j;
  uint32_t* __restrict__ out = row_idx + m * nbr * nbc + col_ptr[m * (nbc + 1) + j];
  int written = 0;
  for (int base = 0; base < nbr; base += 64) {
    const uint8_t v = (base + lane < nbr) ? c[(int64_t)(base + lane) * nbc] : (uint8_t)0;
    const uint64_t nz = __ballot(v != BBM_BLOCK_EMPTY);
    if (v != BBM_BLOCK_EMPTY) out[written + __popcll(nz & ((1ull << lane) - 1ull))] = (uint32_t)(base + lane) | (v == BBM_BLOCK_FULL ? 0x80000000u : 0u);
    written += __popcll(nz);
  }
}

// Split schedule of the column walk: columns with more than T = max(kColSchedMinSplit, 2 * mean entries per non-empty
// column) list entries are cut into ceil(n/T) near-equal parts; work-group 0 scans all Mb*nbc columns for that.
// Work-group 1 + m writes the launch-order records of plane m: columns by list length, longest first (ties: the
// higher column first), each with what a work-group needs to start (column, list position, entries, first entry).
constexpr int kColSchedThreads = 256;

__device__ __forceinline__ int wave_incl_scan(int x, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int up = __shfl_up(x, d);
    if (lane >= d) x += up;
  }
  return x;
}

__global__ __launch_bounds__(kColSchedThreads) void col_sched_kernel(const int32_t* __restrict__ col_ptr,
                                                                    const uint32_t* __restrict__ row_idx, int Mb, int nbr, int nbc,
                                                                    int32_t* __restrict__ sched) {
  constexpr int NWV = kColSchedThreads / 64;
  __shared__ long long tot_s[NWV];
  __shared__ int ne_s[NWV];
  __shared__ int np_s[NWV], cut_s[NWV];
  __shared__ int len_s[bbm::kSchedMaxSortRows];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int C = Mb * nbc;
  if (blockIdx.x > 0) {
    const int m = blockIdx.x - 1;
    int32_t* __restrict__ ord = sched + bbm::kSchedPartBase + (int64_t)bbm::kSchedPartInts * C + (int64_t)bbm::kSchedRowInts * m * nbc;
    const int32_t* __restrict__ cp = col_ptr + (int64_t)m * (nbc + 1);
    const uint32_t* __restrict__ lst = row_idx + (int64_t)m * nbr * nbc;
    const bool sorted = nbc <= bbm::kSchedMaxSortRows;
    if (sorted) {
      for (int j = tid; j < nbc; j += kColSchedThreads) len_s[j] = cp[j + 1] - cp[j];
      __syncthreads();
    }
    for (int j = tid; j < nbc; j += kColSchedThreads) {
      const int pos = cp[j], n = cp[j + 1] - pos;
      int rank = nbc - 1 - j;
      if (sorted) {
        rank = 0;
        for (int x = 0; x < nbc; ++x) {
          const int lx = len_s[x];
          rank += (lx > n || (lx == n && x > j)) ? 1 : 0;
        }
      }
      int32_t* rec = ord + bbm::kSchedRowInts * rank;
      rec[0] = j;
      rec[1] = pos;
      rec[2] = n;
      rec[3] = n > 0 ? (int32_t)lst[pos] : -1;
    }
    return;
  }
  auto count_of = [&](int c) {
    const int m = c / nbc, j = c - m * nbc;
    const int32_t* p = col_ptr + (int64_t)m * (nbc + 1) + j;
    return p[1] - p[0];
  };
  long long total = 0;
  int nonempty = 0;
  for (int c = tid; c < C; c += kColSchedThreads) {
    const int n = count_of(c);
    total += n;
    nonempty += n > 0 ? 1 : 0;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    total += __shfl_xor(total, d);
    nonempty += __shfl_xor(nonempty, d);
  }
  if (lane == 0) {
    tot_s[wave] = total;
    ne_s[wave] = nonempty;
  }
  __syncthreads();
  total = 0;
  nonempty = 0;
  for (int w = 0; w < NWV; ++w) {
    total += tot_s[w];
    nonempty += ne_s[w];
  }
  const int mean = nonempty > 0 ? (int)((total + nonempty - 1) / nonempty) : 0;
  const int T = max(bbm::kColSchedMinSplit, 2 * mean);
  int qbase = 0, rbase = 0;
  for (int c0 = 0; c0 < C; c0 += kColSchedThreads) {
    const int c = c0 + tid;
    const int n = c < C ? count_of(c) : 0;
    const int np = n > T ? (n + T - 1) / T : 0;
    const int cut = np > 0 ? 1 : 0;
    const int inp = wave_incl_scan(np, lane), icut = wave_incl_scan(cut, lane);
    __syncthreads();  // the previous chunk's totals have been read
    if (lane == 63) {
      np_s[wave] = inp;
      cut_s[wave] = icut;
    }
    __syncthreads();
    int q = qbase + inp - np, rho = rbase + icut - cut, chunk_np = 0, chunk_cut = 0;
    for (int w = 0; w < NWV; ++w) {
      if (w < wave) {
        q += np_s[w];
        rho += cut_s[w];
      }
      chunk_np += np_s[w];
      chunk_cut += cut_s[w];
    }
    if (np > 0) {
      const int m = c / nbc, j = c - m * nbc;
      const int first0 = col_ptr[(int64_t)m * (nbc + 1) + j];
      const int chunk = (n + np - 1) / np;
      for (int k = 0; k < np; ++k) {
        int32_t* rec = sched + bbm::kSchedPartBase + (int64_t)bbm::kSchedPartInts * (q + k);
        const int first = first0 + k * chunk;
        rec[0] = c;
        rec[1] = first;
        rec[2] = min(chunk, n - k * chunk);
        rec[3] = k;
        rec[4] = np;
        rec[5] = q;
        rec[6] = rho;
        rec[7] = (int32_t)row_idx[(int64_t)m * nbr * nbc + first];
      }
    }
    qbase += chunk_np;
    rbase += chunk_cut;
  }
  if (tid < bbm::kSchedPartBase) sched[tid] = tid == bbm::kSchedNParts ? qbase : tid == bbm::kSchedSplitT ? T : tid == bbm::kSchedNCutRows ? rbase : 0;
}

}  // namespace

extern "C" __attribute__((visibility("default"))) size_t bbm_col_sched_bytes(int64_t Mb, int64_t nbc) {
  if (Mb < 1 || nbc < 1) return 0;
  return (size_t)(bbm::kSchedPartBase + (bbm::kSchedPartInts + bbm::kSchedRowInts) * Mb * nbc) * sizeof(int32_t);
}

extern "C" __attribute__((visibility("default"))) int bbm_build_col_index(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc,
                                                                         int32_t* col_ptr, uint32_t* row_idx, int32_t* col_sched,
                                                                         void* stream) {
  using namespace bbm;
  clear_error();
  if (!blk_class || !col_ptr || !row_idx) return fail(BBM_EINVAL, "bbm_build_col_index: blk_class, col_ptr, row_idx must not be NULL");
  if (Mb < 1 || nbr < 1 || nbc < 1)
    return fail(BBM_EINVAL, "bbm_build_col_index: Mb=%lld, nbr=%lld, nbc=%lld must be >= 1", (long long)Mb, (long long)nbr, (long long)nbc);
  if (!aligned(col_ptr, 4) || !aligned(row_idx, 4)) return fail(BBM_EINVAL, "bbm_build_col_index: col_ptr, row_idx must be 4-byte aligned");
  if (col_sched && !aligned(col_sched, 32)) return fail(BBM_EINVAL, "bbm_build_col_index: col_sched must be 32-byte aligned");
  if (col_sched && Mb * nbc >= (1ll << 24)) return fail(BBM_EINVAL, "bbm_build_col_index: Mb*nbc must be below 2^24 for a schedule");
  if (nbr * nbc >= (1ll << 31) || Mb >= (1ll << 31)) return fail(BBM_EINVAL, "bbm_build_col_index: nbr*nbc and Mb must be below 2^31");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (nbr <= kColOneKernelRows) {
    col_index_kernel<<<(unsigned)Mb, kColThreads, 0, st>>>(blk_class, (int)nbr, (int)nbc, col_ptr, row_idx);
  } else {
    if (ceil_div(Mb * nbc, kColWaves) >= (1ll << 31)) return fail(BBM_EINVAL, "bbm_build_col_index: Mb*nbc too large");
    const unsigned grid = (unsigned)ceil_div(Mb * nbc, kColWaves);
    col_count_kernel<<<grid, kColWaves * 64, 0, st>>>(blk_class, Mb, (int)nbr, (int)nbc, col_ptr);
    col_scan_kernel<<<(unsigned)Mb, 64, 0, st>>>((int)nbc, col_ptr);
    col_fill_kernel<<<grid, kColWaves * 64, 0, st>>>(blk_class, Mb, (int)nbr, (int)nbc, col_ptr, row_idx);
  }
  int rc = launch_status("bbm_build_col_index");
  if (rc != BBM_OK || !col_sched) return rc;
  col_sched_kernel<<<(unsigned)(1 + Mb), kColSchedThreads, 0, static_cast<hipStream_t>(stream)>>>(col_ptr, row_idx, (int)Mb, (int)nbr, (int)nbc, col_sched);
  return launch_status("bbm_build_col_index (schedule)");
}
