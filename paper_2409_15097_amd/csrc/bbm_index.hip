// Stage 1b / 1c: run index of the "Dense" variant (paper Sec. 4: total_ones / offset per block row) and the
// compact per-row list of non-zero blocks.  Both read only the small [Mb][nbr][nbc] class matrix; one
// wavefront owns one block row and works on 64 classes at a time through wave-wide ballots.
#include "bbm_internal.h"

namespace {

constexpr int kWavesPerWG = 4;

__device__ __forceinline__ int ctz64(uint64_t x) { return x ? __builtin_ctzll(x) : 64; }

// One wave per block row.  Longest run of FULL blocks (leftmost on ties) and the span of non-zero blocks.
__global__ __launch_bounds__(kWavesPerWG * 64) void runs_kernel(const uint8_t* __restrict__ cls, int64_t rows_total,
                                                                int64_t nbc, int32_t* __restrict__ offset,
                                                                int32_t* __restrict__ total_ones,
                                                                int32_t* __restrict__ nz_lo, int32_t* __restrict__ nz_hi,
                                                                int32_t* __restrict__ nz_cnt) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * kWavesPerWG + (threadIdx.x >> 6);
  if (row >= rows_total) return;
  const uint8_t* c = cls + row * nbc;

  int best_len = 0, best_start = 0;  // longest finished run so far
  int cur_len = 0, cur_start = 0;    // run that touches the end of the previous chunk (0 = none)
  int lo = 0, hi = 0, cnt = 0;
  for (int64_t base = 0; base < nbc; base += 64) {
    const uint8_t v = (base + lane < nbc) ? c[base + lane] : (uint8_t)0;
    uint64_t full = __ballot(v == BBM_BLOCK_FULL);
    const uint64_t nz = __ballot(v != BBM_BLOCK_EMPTY);
    if (nz) {
      if (cnt == 0) lo = (int)base + ctz64(nz);
      hi = (int)base + 64 - __builtin_clzll(nz);
      cnt += __popcll(nz);
    }
    if (cur_len > 0) {  // continue the run that reached the chunk boundary
      const int ones = ctz64(~full);
      cur_len += ones;
      if (ones == 64) continue;
      if (cur_len > best_len) { best_len = cur_len; best_start = cur_start; }
      cur_len = 0;
      full &= ~((1ull << ones) - 1ull);
    }
    while (full) {
      const int s = ctz64(full);
      const int ones = ctz64(~(full >> s));  // full >> s has zeros shifted in, so ones <= 64 - s
      if (s + ones == 64) {                  // run reaches the chunk end: decide when it ends
        cur_start = (int)base + s;
        cur_len = ones;
        break;
      }
      if (ones > best_len) { best_len = ones; best_start = (int)base + s; }
      full &= ~(((1ull << ones) - 1ull) << s);
    }
  }
  if (cur_len > best_len) { best_len = cur_len; best_start = cur_start; }
  if (lane == 0) {
    offset[row] = best_start;
    total_ones[row] = best_len;
    nz_lo[row] = lo;
    nz_hi[row] = hi;
    nz_cnt[row] = cnt;
  }
}

// Pass 1 of the list: row_ptr[m][i+1] <- number of non-zero blocks of row i (one wave per row).
__global__ __launch_bounds__(kWavesPerWG * 64) void list_count_kernel(const uint8_t* __restrict__ cls, int64_t Mb,
                                                                      int64_t nbr, int64_t nbc,
                                                                      int32_t* __restrict__ row_ptr) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * kWavesPerWG + (threadIdx.x >> 6);
  if (row >= Mb * nbr) return;
  const uint8_t* c = cls + row * nbc;
  int cnt = 0;
  for (int64_t base = 0; base < nbc; base += 64) {
    const uint8_t v = (base + lane < nbc) ? c[base + lane] : (uint8_t)0;
    cnt += __popcll(__ballot(v != BBM_BLOCK_EMPTY));
  }
  const int64_t m = row / nbr, i = row - m * nbr;
  if (lane == 0) row_ptr[m * (nbr + 1) + i + 1] = cnt;
}

// Pass 2: in-place inclusive scan of row_ptr[m][1..nbr], one wave per plane, 64 rows per step.
__global__ __launch_bounds__(64) void list_scan_kernel(int64_t nbr, int32_t* __restrict__ row_ptr) {
  const int lane = threadIdx.x;
  int32_t* p = row_ptr + (int64_t)blockIdx.x * (nbr + 1);
  int carry = 0;
  for (int64_t base = 0; base < nbr; base += 64) {
    int x = (base + lane < nbr) ? p[base + lane + 1] : 0;
    for (int s = 1; s < 64; s <<= 1) {
      const int y = __shfl_up(x, s);
      if (lane >= s) x += y;
    }
    x += carry;
    if (base + lane < nbr) p[base + lane + 1] = x;
    carry = __shfl(x, 63);
  }
  if (lane == 0) p[0] = 0;
}

// Pass 3: write the ascending list of each row at row_ptr[m][i] (one wave per row).
__global__ __launch_bounds__(kWavesPerWG * 64) void list_fill_kernel(const uint8_t* __restrict__ cls, int64_t Mb,
                                                                     int64_t nbr, int64_t nbc,
                                                                     const int32_t* __restrict__ row_ptr,
                                                                     uint32_t* __restrict__ col_idx) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * kWavesPerWG + (threadIdx.x >> 6);
  if (row >= Mb * nbr) return;
  const int64_t m = row / nbr, i = row - m * nbr;
  const uint8_t* c = cls + row * nbc;
  uint32_t* out = col_idx + m * nbr * nbc + row_ptr[m * (nbr + 1) + i];
  int written = 0;
  for (int64_t base = 0; base < nbc; base += 64) {
    const uint8_t v = (base + lane < nbc) ? c[base + lane] : (uint8_t)0;
    const uint64_t nz = __ballot(v != BBM_BLOCK_EMPTY);
    if (v != BBM_BLOCK_EMPTY) {
      const int pos = written + __popcll(nz & ((1ull << lane) - 1ull));
      out[pos] = (uint32_t)(base + lane) | (v == BBM_BLOCK_FULL ? 0x80000000u : 0u);
    }
    written += __popcll(nz);
  }
}

}  // namespace

extern "C" __attribute__((visibility("default"))) int bbm_build_runs(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, int32_t* offset,
                              int32_t* total_ones, int32_t* nz_lo, int32_t* nz_hi, int32_t* nz_cnt, void* stream) {
  using namespace bbm;
  clear_error();
  if (!blk_class || !offset || !total_ones || !nz_lo || !nz_hi || !nz_cnt)
    return fail(BBM_EINVAL, "bbm_build_runs: NULL pointer argument");
  if (Mb < 1 || nbr < 1 || nbc < 1)
    return fail(BBM_EINVAL, "bbm_build_runs: Mb=%lld, nbr=%lld, nbc=%lld must be >= 1", (long long)Mb, (long long)nbr, (long long)nbc);
  if (nbc > (1ll << 30) || Mb * nbr > (1ll << 31) * kWavesPerWG - 1)
    return fail(BBM_EUNSUPPORTED, "bbm_build_runs: index too large");
  const int64_t rows = Mb * nbr;
  runs_kernel<<<(unsigned)ceil_div(rows, kWavesPerWG), kWavesPerWG * 64, 0, static_cast<hipStream_t>(stream)>>>(
      blk_class, rows, nbc, offset, total_ones, nz_lo, nz_hi, nz_cnt);
  return launch_status("bbm_build_runs");
}

extern "C" __attribute__((visibility("default"))) int bbm_build_sparse_index(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc,
                                      int32_t* row_ptr, uint32_t* col_idx, void* stream) {
  using namespace bbm;
  clear_error();
  if (!blk_class || !row_ptr || !col_idx) return fail(BBM_EINVAL, "bbm_build_sparse_index: NULL pointer argument");
  if (Mb < 1 || nbr < 1 || nbc < 1)
    return fail(BBM_EINVAL, "bbm_build_sparse_index: Mb=%lld, nbr=%lld, nbc=%lld must be >= 1", (long long)Mb, (long long)nbr, (long long)nbc);
  if (nbr * nbc >= (1ll << 31) || Mb > (1ll << 30) || Mb * nbr > (1ll << 31) * kWavesPerWG - 1)
    return fail(BBM_EUNSUPPORTED, "bbm_build_sparse_index: nbr*nbc=%lld must be < 2^31", (long long)(nbr * nbc));
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned grid = (unsigned)ceil_div(Mb * nbr, kWavesPerWG);
  list_count_kernel<<<grid, kWavesPerWG * 64, 0, s>>>(blk_class, Mb, nbr, nbc, row_ptr);
  int rc = launch_status("bbm_build_sparse_index(count)");
  if (rc) return rc;
  list_scan_kernel<<<(unsigned)Mb, 64, 0, s>>>(nbr, row_ptr);
  rc = launch_status("bbm_build_sparse_index(scan)");
  if (rc) return rc;
  list_fill_kernel<<<grid, kWavesPerWG * 64, 0, s>>>(blk_class, Mb, nbr, nbc, row_ptr, col_idx);
  return launch_status("bbm_build_sparse_index(fill)");
}
