// Stage 1b / 1c: run index of the "Dense" variant (paper Sec. 4: total_ones / offset per block row) and the
// compact per-row list of non-zero blocks.  Both read only the small [Mb][nbr][nbc] class matrix; one
// wavefront owns one block row and works on 64 classes at a time through wave-wide ballots.
#include "bbm_internal.h"

namespace {

constexpr int kWavesPerWG = 4;

__device__ __forceinline__ int ctz64(uint64_t x) { return x ? __builtin_ctzll(x) : 64; }

// Longest run of FULL blocks of one block row (leftmost on ties) and the span of its non-zero blocks, fed 64 block
// columns at a time in ascending order (bit t of `full` / `nz` = block column base + t).
struct RunScan {
  int best_len = 0, best_start = 0;  // longest finished run so far
  int cur_len = 0, cur_start = 0;    // run that touches the end of the previous chunk (0 = none)
  int lo = 0, hi = 0, cnt = 0;
  __device__ __forceinline__ void feed(uint64_t full, uint64_t nz, int base) {
    if (nz) {
      if (cnt == 0) lo = base + ctz64(nz);
      hi = base + 64 - __builtin_clzll(nz);
      cnt += __popcll(nz);
    }
    if (cur_len > 0) {  // continue the run that reached the chunk boundary
      const int ones = ctz64(~full);
      cur_len += ones;
      if (ones == 64) return;
      if (cur_len > best_len) { best_len = cur_len; best_start = cur_start; }
      cur_len = 0;
      full &= ~((1ull << ones) - 1ull);
    }
    while (full) {
      const int s = ctz64(full);
      const int ones = ctz64(~(full >> s));  // full >> s has zeros shifted in, so ones <= 64 - s
      if (s + ones == 64) {                  // run reaches the chunk end: decide when it ends
        cur_start = base + s;
        cur_len = ones;
        return;
      }
      if (ones > best_len) { best_len = ones; best_start = base + s; }
      full &= ~(((1ull << ones) - 1ull) << s);
    }
  }
  __device__ __forceinline__ void finish() {
    if (cur_len > best_len) { best_len = cur_len; best_start = cur_start; }
  }
};

// Exclusive prefix sum over the 64 lanes with data-parallel-primitive moves (register to register; a shuffle goes
// through LDS): shifts by 1, 2, 4, 8 inside each row of 16 lanes (a lane without a source adds 0), then lane 15 of a
// row added to the next row (rows 1 and 3), then lane 31 to rows 2 and 3.
__device__ __forceinline__ int wave_excl_scan(int x, int /*lane*/) {
  int incl = x;
  incl += __builtin_amdgcn_update_dpp(0, incl, 0x111, 0xf, 0xf, false);  // row_shr:1
  incl += __builtin_amdgcn_update_dpp(0, incl, 0x112, 0xf, 0xf, false);  // row_shr:2
  incl += __builtin_amdgcn_update_dpp(0, incl, 0x114, 0xf, 0xf, false);  // row_shr:4
  incl += __builtin_amdgcn_update_dpp(0, incl, 0x118, 0xf, 0xf, false);  // row_shr:8
  incl += __builtin_amdgcn_update_dpp(0, incl, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1, 3
  incl += __builtin_amdgcn_update_dpp(0, incl, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2, 3
  return incl - x;
}

// One wave per block row.  With `row_ptr` (rows per plane: nbr) the row's count of non-zero blocks is also left at
// row_ptr[m][i+1], which is pass 1 of the list: the index stage in one call then needs no list_count_kernel.
__global__ __launch_bounds__(kWavesPerWG * 64) void runs_kernel(const uint8_t* __restrict__ cls, int64_t rows_total,
                                                                int64_t nbc, int32_t* __restrict__ offset,
                                                                int32_t* __restrict__ total_ones,
                                                                int32_t* __restrict__ nz_lo, int32_t* __restrict__ nz_hi,
                                                                int32_t* __restrict__ nz_cnt, int32_t* __restrict__ row_ptr,
                                                                int64_t nbr) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * kWavesPerWG + (threadIdx.x >> 6);
  if (row >= rows_total) return;
  const uint8_t* c = cls + row * nbc;
  RunScan rs;
  for (int64_t base = 0; base < nbc; base += 64) {
    const uint8_t v = (base + lane < nbc) ? c[base + lane] : (uint8_t)0;
    rs.feed(__ballot(v == BBM_BLOCK_FULL), __ballot(v != BBM_BLOCK_EMPTY), (int)base);
  }
  rs.finish();
  if (lane == 0) {
    offset[row] = rs.best_start;
    total_ones[row] = rs.best_len;
    nz_lo[row] = rs.lo;
    nz_hi[row] = rs.hi;
    nz_cnt[row] = rs.cnt;
    if (row_ptr) {
      const int64_t m = row / nbr, i = row - m * nbr;
      row_ptr[m * (nbr + 1) + i + 1] = rs.cnt;
    }
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
    x += wave_excl_scan(x, lane);
    x += carry;
    if (base + lane < nbr) p[base + lane + 1] = x;
    carry = __shfl(x, 63);
  }
  if (lane == 0) p[0] = 0;
}

// Pass 3: write the ascending list of each row at row_ptr[m][i] (one wave per row).  With `counts` ([Mb][nbr] list
// lengths, as the runs kernel leaves them in nz_cnt) pass 2 is done here as well: the wave adds up the counts of the
// rows above its own -- a few hundred integers -- and writes its entry of row_ptr itself.
__global__ __launch_bounds__(kWavesPerWG * 64) void list_fill_kernel(const uint8_t* __restrict__ cls, int64_t Mb,
                                                                     int64_t nbr, int64_t nbc,
                                                                     int32_t* __restrict__ row_ptr,
                                                                     const int32_t* __restrict__ counts,
                                                                     uint32_t* __restrict__ col_idx) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * kWavesPerWG + (threadIdx.x >> 6);
  if (row >= Mb * nbr) return;
  const int64_t m = row / nbr, i = row - m * nbr;
  const uint8_t* c = cls + row * nbc;
  int start;
  if (counts) {
    const int32_t* cp = counts + m * nbr;
    int part = 0;
    for (int64_t b = lane; b < i; b += 64) part += cp[b];
    start = __builtin_amdgcn_readlane(wave_excl_scan(part, lane) + part, 63);
    if (lane == 0) {
      row_ptr[m * (nbr + 1) + i] = start;
      if (i == nbr - 1) row_ptr[m * (nbr + 1) + nbr] = start + cp[i];
    }
  } else {
    start = row_ptr[m * (nbr + 1) + i];
  }
  uint32_t* out = col_idx + m * nbr * nbc + start;
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

// Rows per launch-order group: neighbouring rows are kept together only while rows are short (split threshold at its
// floor, i.e. mean list length <= 16); with long rows the plain longest-first order balances the tail better.
__device__ __forceinline__ int launch_group_rows(int T) { return T == bbm::kSchedMinSplit ? bbm::kSchedGroupRows : 1; }

// Position of block row i in the launch order of its plane.  len[0 .. nbr) = list lengths of the plane's rows,
// gmax[0 .. ceil(nbr/gsz)) = longest list of every group of gsz consecutive rows.  Order: the group holding the longest
// row first (ties: higher rows first); inside a group the longest row first (ties: higher row first).
__device__ __forceinline__ int launch_rank(const int* len, const int* gmax, int nbr, int gsz, int i) {
  const int ng = (nbr + gsz - 1) / gsz, g = i / gsz;
  const int mine = gmax[g];
  int before = 0;  // groups that go first
  for (int gg = 0; gg < ng; ++gg) {
    const int t = gmax[gg];
    before += (t > mine) || (t == mine && gg > g);
  }
  int rank = before * gsz;
  // the last group may be short; it is among the groups that go first iff its turn comes before g's
  const int last = ng - 1, last_rows = nbr - last * gsz;
  if (last != g && (gmax[last] > mine || gmax[last] == mine)) rank -= gsz - last_rows;
  const int c = len[i];
  for (int j = g * gsz; j < min(nbr, (g + 1) * gsz); ++j) rank += (len[j] > c) || (len[j] == c && j > i);
  return rank;
}

// Sum over the 64 lanes, returned in every lane.
__device__ __forceinline__ int wave_sum(int x) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d);
  return x;
}

// list_fill_kernel and sched_kernel in one launch, for index stages that already have every row's list length
// (`counts` = the runs kernel's nz_cnt, [Mb][nbr]) and at most kFuseSchedRows block rows over all planes: the wave that
// fills a row's list also writes the row's launch-order record, and the records of its parts if the schedule cuts the row.
// Everything a wave needs beyond its own row -- the split threshold (a mean over all rows), the parts and cut rows
// before its own, its rank among the rows of its plane -- it counts itself from `counts` (a few hundred to a few
// thousand integers), so no wave waits for another.  Same schedule, bit for bit, as sched_kernel writes.
constexpr int64_t kFuseSchedRows = 4096;
__global__ __launch_bounds__(kWavesPerWG * 64) void list_fill_sched_kernel(const uint8_t* __restrict__ cls, int Mb, int nbr, int nbc,
                                                                           int32_t* __restrict__ row_ptr,
                                                                           const int32_t* __restrict__ counts,
                                                                           uint32_t* __restrict__ col_idx, int32_t* __restrict__ sched) {
  using namespace bbm;
  const int lane = threadIdx.x & 63;
  const int row = (int)blockIdx.x * kWavesPerWG + (int)(threadIdx.x >> 6);
  const int nrows = Mb * nbr;
  if (row >= nrows) return;
  const int m = row / nbr, i = row - m * nbr;
  const int32_t* cp = counts + (int64_t)m * nbr;
  const int c = cp[i];

  // position of the row's list in its plane, and the totals the split threshold is made of
  int above = 0, total = 0, nonempty = 0;
  for (int b = lane; b < i; b += 64) above += cp[b];
  for (int b = lane; b < nrows; b += 64) {
    const int x = counts[b];
    total += x;
    nonempty += x > 0 ? 1 : 0;
  }
  const int start = wave_sum(above);
  total = wave_sum(total);
  nonempty = wave_sum(nonempty);
  const int mean = nonempty > 0 ? (total + nonempty - 1) / nonempty : 0;
  const int T = max(kSchedMinSplit, 2 * mean);
  if (lane == 0) {
    row_ptr[(int64_t)m * (nbr + 1) + i] = start;
    if (i == nbr - 1) row_ptr[(int64_t)m * (nbr + 1) + nbr] = start + c;
  }

  // parts and cut rows: before this row (rows in (plane, block row) order), and in all
  int q = 0, rho = 0, all_parts = 0, all_cut = 0;
  for (int b = lane; b < nrows; b += 64) {
    const int x = counts[b];
    const int np_b = x > T ? (x + T - 1) / T : 0;
    all_parts += np_b;
    all_cut += np_b > 0 ? 1 : 0;
    if (b < row) {
      q += np_b;
      rho += np_b > 0 ? 1 : 0;
    }
  }
  q = wave_sum(q);
  rho = wave_sum(rho);
  if (row == 0) {
    all_parts = wave_sum(all_parts);
    all_cut = wave_sum(all_cut);
    if (lane < kSchedPartBase)
      sched[lane] = lane == kSchedNParts ? all_parts : lane == kSchedSplitT ? T : lane == kSchedNCutRows ? all_cut : 0;
  }
  const int np = c > T ? (c + T - 1) / T : 0;
  const int chunk = np > 0 ? (c + np - 1) / np : 1;
  int32_t* const parts = sched + kSchedPartBase + (int64_t)kSchedPartInts * q;
  for (int k = lane; k < np; k += 64) {
    int32_t* rec = parts + kSchedPartInts * k;
    rec[0] = row;
    rec[1] = start + k * chunk;
    rec[2] = min(chunk, c - k * chunk);
    rec[3] = k;
    rec[4] = np;
    rec[5] = q;
    rec[6] = rho;
  }

  // the list; the lane that writes the entry a part starts with also leaves it in the part's record
  const uint8_t* cl = cls + (int64_t)row * nbc;
  uint32_t* out = col_idx + (int64_t)m * nbr * nbc + start;
  int written = 0, first = -1;
  for (int base = 0; base < nbc; base += 64) {
    const uint8_t v = (base + lane < nbc) ? cl[base + lane] : (uint8_t)0;
    const uint64_t nz = __ballot(v != BBM_BLOCK_EMPTY);
    const uint64_t full = __ballot(v == BBM_BLOCK_FULL);
    if (written == 0 && nz != 0) {  // the row's first entry (this happens once: written > 0 from here on)
      const int bit = ctz64(nz);
      first = (int)((uint32_t)(base + bit) | (((full >> bit) & 1ull) ? 0x80000000u : 0u));
    }
    if (v != BBM_BLOCK_EMPTY) {
      const int pos = written + __popcll(nz & ((1ull << lane) - 1ull));
      const uint32_t entry = (uint32_t)(base + lane) | (v == BBM_BLOCK_FULL ? 0x80000000u : 0u);
      out[pos] = entry;
      if (np > 0 && pos % chunk == 0 && pos / chunk < np) parts[kSchedPartInts * (pos / chunk) + 7] = (int32_t)entry;
    }
    written += __popcll(nz);
  }

  // launch-order record: rank among the rows of the plane (launch_rank's order, counted over the lanes)
  const int gsz = launch_group_rows(T);
  const int ng = (nbr + gsz - 1) / gsz, g = i / gsz;
  auto group_max = [&](int gg) {
    int t = 0;
    for (int j = gg * gsz; j < min(nbr, (gg + 1) * gsz); ++j) t = max(t, cp[j]);
    return t;
  };
  const int mine = group_max(g);
  int before = 0;
  for (int gg = lane; gg < ng; gg += 64) {
    const int t = group_max(gg);
    before += (t > mine || (t == mine && gg > g)) ? 1 : 0;
  }
  before = wave_sum(before);
  int rank = before * gsz;
  const int last = ng - 1, last_rows = nbr - last * gsz;
  if (last != g && group_max(last) >= mine) rank -= gsz - last_rows;
  for (int j = g * gsz; j < min(nbr, (g + 1) * gsz); ++j) rank += (cp[j] > c || (cp[j] == c && j > i)) ? 1 : 0;
  if (lane == 0)
    reinterpret_cast<int4*>(sched + sched_order_base(Mb, nbr))[(int64_t)m * nbr + rank] = make_int4(i, start, c, first);
}

// Split schedule of LIST mode (layout in bbm_internal.h).  Work-group 0 writes the header and the parts table: every
// thread owns a contiguous range of block rows; pass 1 counts, per thread, the parts and the cut rows; an exclusive
// scan over the threads turns the counts into positions; pass 2 writes the parts in (row, part) order, so the
// result does not depend on the thread count.  Work-group 1 + m writes the row records of plane m in launch order,
// ranking by counting over the list lengths staged in LDS.
constexpr int kSchedThreads = 256;

__global__ __launch_bounds__(kSchedThreads) void sched_kernel(const int32_t* __restrict__ row_ptr,
                                                              const uint32_t* __restrict__ col_idx, int Mb, int nbr,
                                                              int64_t plane_entries, int32_t* __restrict__ sched) {
  using namespace bbm;
  __shared__ int pre[2][kSchedThreads + 1];
  __shared__ int red[2][kSchedThreads];
  __shared__ int len_s[kSchedMaxSortRows];
  __shared__ int gmax_s[kSchedMaxSortRows];
  const int tid = threadIdx.x;
  const int nrows = Mb * nbr;
  const int per = (nrows + kSchedThreads - 1) / kSchedThreads;
  const int r_lo = min(nrows, tid * per), r_hi = min(nrows, r_lo + per);
  auto first_entry = [&](int r) {
    const int m = r / nbr, i = r - m * nbr;
    return row_ptr + (int64_t)m * (nbr + 1) + i;
  };

  // split threshold from the mean list length of the non-empty rows (every work-group needs it)
  int total = 0, nonempty = 0;
  for (int r = r_lo; r < r_hi; ++r) {
    const int32_t* rp = first_entry(r);
    const int c = rp[1] - rp[0];
    total += c;
    nonempty += c > 0;
  }
  red[0][tid] = total;
  red[1][tid] = nonempty;
  __syncthreads();
  for (int s = kSchedThreads / 2; s > 0; s >>= 1) {
    if (tid < s) {
      red[0][tid] += red[0][tid + s];
      red[1][tid] += red[1][tid + s];
    }
    __syncthreads();
  }
  total = red[0][0];
  nonempty = red[1][0];
  const int mean = nonempty > 0 ? (total + nonempty - 1) / nonempty : 0;
  const int T = max(kSchedMinSplit, 2 * mean);

  if (blockIdx.x > 0) {
    const int m = blockIdx.x - 1;
    const int32_t* rp = row_ptr + (int64_t)m * (nbr + 1);
    const uint32_t* list = col_idx + (int64_t)m * plane_entries;
    int4* rec = reinterpret_cast<int4*>(sched + sched_order_base(Mb, nbr)) + (int64_t)m * nbr;
    const bool sorted = nbr <= kSchedMaxSortRows;
    const int gsz = launch_group_rows(T);
    if (sorted) {
      for (int j = tid; j < nbr; j += kSchedThreads) len_s[j] = rp[j + 1] - rp[j];
      __syncthreads();
      for (int g = tid; g * gsz < nbr; g += kSchedThreads) {
        int t = 0;
        for (int j = g * gsz; j < min(nbr, (g + 1) * gsz); ++j) t = max(t, len_s[j]);
        gmax_s[g] = t;
      }
      __syncthreads();
    }
    for (int i = tid; i < nbr; i += kSchedThreads) {
      const int p0 = rp[i], c = rp[i + 1] - p0;
      const int rank = sorted ? launch_rank(len_s, gmax_s, nbr, gsz, i) : nbr - 1 - i;
      rec[rank] = make_int4(i, p0, c, c > 0 ? (int)list[p0] : -1);
    }
    return;
  }

  int nparts = 0, ncut = 0;
  for (int r = r_lo; r < r_hi; ++r) {
    const int32_t* rp = first_entry(r);
    const int c = rp[1] - rp[0];
    if (c > T) {
      nparts += (c + T - 1) / T;
      ncut += 1;
    }
  }
  // exclusive scan over the threads: inside each wave with register moves, then the four wave totals through LDS
  const int lane = tid & 63, wave = tid >> 6;
  const int q_in_wave = wave_excl_scan(nparts, lane), rho_in_wave = wave_excl_scan(ncut, lane);
  if (lane == 63) {
    pre[0][wave] = q_in_wave + nparts;
    pre[1][wave] = rho_in_wave + ncut;
  }
  __syncthreads();
  int q = q_in_wave, rho = rho_in_wave, all_parts = 0, all_cut = 0;
  for (int w = 0; w < kSchedThreads / 64; ++w) {
    q += w < wave ? pre[0][w] : 0;
    rho += w < wave ? pre[1][w] : 0;
    all_parts += pre[0][w];
    all_cut += pre[1][w];
  }
  if (tid == 0) {
    sched[kSchedNParts] = all_parts;
    sched[kSchedSplitT] = T;
    sched[kSchedNCutRows] = all_cut;
    for (int x = 3; x < kSchedPartBase; ++x) sched[x] = 0;
  }
  for (int r = r_lo; r < r_hi; ++r) {
    const int32_t* rp = first_entry(r);
    const int c = rp[1] - rp[0];
    if (c <= T) continue;
    const uint32_t* list = col_idx + (int64_t)(r / nbr) * plane_entries;
    const int np = (c + T - 1) / T;
    const int chunk = (c + np - 1) / np;
    for (int k = 0; k < np; ++k) {
      int32_t* rec = sched + kSchedPartBase + (int64_t)kSchedPartInts * (q + k);
      rec[0] = r;
      rec[1] = rp[0] + k * chunk;
      rec[2] = min(chunk, c - k * chunk);
      rec[3] = k;
      rec[4] = np;
      rec[5] = q;
      rec[6] = rho;
      rec[7] = (int32_t)list[rp[0] + k * chunk];
    }
    q += np;
    rho += 1;
  }
}

// The same products for the smallest class matrices -- at most 64 block rows per plane, at most 256 block columns in
// whole 16-byte groups, at most 16 planes (4 planes of a 4096 x 4096 mask in 128 x 64 or 64 x 64 tiles) -- with one
// WAVE per plane and one LANE per block row: a lane reads its row as 16-byte words and turns it into a non-zero and a
// full bit mask in registers, so counting, run search and list positions need no ballots and no LDS; row_ptr is a
// shuffle scan over the lanes.  Only the split threshold (a mean over all planes) and the launch-order ranks cross
// lanes through LDS, behind two barriers.
constexpr int kTinyMaxPlanes = 16, kTinyMaxRows = 64, kTinyMaxChunks = 4;

// 16 class bytes -> 16 bits: bit t = (byte t != 0) in the low half, (byte t == BBM_BLOCK_FULL) in the high half.
__device__ __forceinline__ uint32_t class_bits16(uint4 x) {
  auto nz4 = [](uint32_t w) {  // 4 bytes -> 4 bits (bit t = byte t non-zero)
    const uint32_t y = (((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) | w) & 0x80808080u;
    return (((y >> 7) * 0x00204081u) >> 21) & 0xfu;
  };
  const uint32_t f = 0x01010101u * BBM_BLOCK_FULL;
  const uint32_t nz = nz4(x.x) | (nz4(x.y) << 4) | (nz4(x.z) << 8) | (nz4(x.w) << 12);
  const uint32_t ne = nz4(x.x ^ f) | (nz4(x.y ^ f) << 4) | (nz4(x.z ^ f) << 8) | (nz4(x.w ^ f) << 12);  // byte != FULL
  return nz | ((~ne & 0xffffu) << 16);
}


__global__ __launch_bounds__(kTinyMaxPlanes * 64) void tiny_index_kernel(const uint8_t* __restrict__ cls, int Mb, int nbr,
                                                                        int nbc, int32_t* __restrict__ row_ptr,
                                                                        uint32_t* __restrict__ col_idx,
                                                                        int32_t* __restrict__ sched,
                                                                        int32_t* __restrict__ offset,
                                                                        int32_t* __restrict__ total_ones,
                                                                        int32_t* __restrict__ nz_lo,
                                                                        int32_t* __restrict__ nz_hi,
                                                                        int32_t* __restrict__ nz_cnt) {
  using namespace bbm;
  __shared__ int tot_s[kTinyMaxPlanes][2];   // per plane: list entries, non-empty rows
  __shared__ int part_s[kTinyMaxPlanes][2];  // per plane: parts, cut rows
  __shared__ int len_s[kTinyMaxPlanes][kTinyMaxRows];
  __shared__ int gmax_s[kTinyMaxPlanes][kTinyMaxRows];
  const int lane = threadIdx.x & 63;
  const int m = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // plane of this wave
  const int i = lane;                                              // block row of this lane
  const bool live = i < nbr;
  const int CH = (nbc + 63) / 64;

  // ---- the row as bit masks
  uint64_t nz[kTinyMaxChunks], full[kTinyMaxChunks];
  {
    const uint4* rowp = reinterpret_cast<const uint4*>(cls + ((int64_t)m * nbr + (live ? i : 0)) * nbc);
    const int words = nbc / 16;
    uint4 w[kTinyMaxChunks * 4];
#pragma unroll
    for (int t = 0; t < kTinyMaxChunks * 4; ++t) w[t] = (live && t < words) ? rowp[t] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int ch = 0; ch < kTinyMaxChunks; ++ch) {
      nz[ch] = full[ch] = 0;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint32_t b = class_bits16(w[4 * ch + t]);
        nz[ch] |= (uint64_t)(b & 0xffffu) << (16 * t);
        full[ch] |= (uint64_t)(b >> 16) << (16 * t);
      }
    }
  }
  int c = 0;
#pragma unroll
  for (int ch = 0; ch < kTinyMaxChunks; ++ch) c += __popcll(nz[ch]);

  // ---- list: position by a scan over the rows of the plane, entries written row by row.  A cross-lane step costs
  // an LDS round trip, so two quantities share each scan (counts stay below 2^16: at most 64 rows of at most 256
  // entries) and totals are read from lane 63 of the scan instead of being reduced again.
  const int packed_c = c | ((c > 0 ? 1 : 0) << 16);
  const int scan_c = wave_excl_scan(packed_c, lane);
  const int start = scan_c & 0xffff;
  if (live) {
    row_ptr[(int64_t)m * (nbr + 1) + i] = start;
    if (i == nbr - 1) row_ptr[(int64_t)m * (nbr + 1) + nbr] = start + c;
    uint32_t* out = col_idx + (int64_t)m * nbr * nbc + start;
#pragma unroll
    for (int ch = 0; ch < kTinyMaxChunks; ++ch) {
      uint64_t x = nz[ch];
      while (x) {
        const int b = ctz64(x);
        *out++ = (uint32_t)(64 * ch + b) | (((full[ch] >> b) & 1ull) ? 0x80000000u : 0u);
        x &= x - 1;
      }
    }
    if (offset) {  // run index
      RunScan rs;
      for (int ch = 0; ch < CH; ++ch) rs.feed(full[ch], nz[ch], 64 * ch);
      rs.finish();
      offset[m * nbr + i] = rs.best_start;
      total_ones[m * nbr + i] = rs.best_len;
      nz_lo[m * nbr + i] = rs.lo;
      nz_hi[m * nbr + i] = rs.hi;
      nz_cnt[m * nbr + i] = rs.cnt;
    }
  }
  if (!sched) return;

  // ---- schedule (same definition as sched_kernel)
  const int last_c = __builtin_amdgcn_readlane(scan_c + packed_c, 63);
  const int plane_total = last_c & 0xffff, plane_nonempty = last_c >> 16;
  if (lane == 0) {
    tot_s[m][0] = plane_total;
    tot_s[m][1] = plane_nonempty;
  }
  if (live) len_s[m][i] = c;
  __syncthreads();
  int total = 0, nonempty = 0;
  for (int p = 0; p < Mb; ++p) {
    total += tot_s[p][0];
    nonempty += tot_s[p][1];
  }
  const int mean = nonempty > 0 ? (total + nonempty - 1) / nonempty : 0;
  const int T = max(kSchedMinSplit, 2 * mean);
  const int np = c > T ? (c + T - 1) / T : 0;
  const int packed_np = np | ((np > 0 ? 1 : 0) << 16);
  const int scan_np = wave_excl_scan(packed_np, lane);
  const int q_in_plane = scan_np & 0xffff, rho_in_plane = scan_np >> 16;
  const int last_np = __builtin_amdgcn_readlane(scan_np + packed_np, 63);
  const int plane_parts = last_np & 0xffff, plane_cut = last_np >> 16;
  if (lane == 0) {
    part_s[m][0] = plane_parts;
    part_s[m][1] = plane_cut;
  }
  const int gsz = launch_group_rows(T), ngp = (nbr + gsz - 1) / gsz;
  if (lane < ngp) {
    int t = 0;
    for (int j = lane * gsz; j < min(nbr, (lane + 1) * gsz); ++j) t = max(t, len_s[m][j]);
    gmax_s[m][lane] = t;
  }
  __syncthreads();
  int q = q_in_plane, rho = rho_in_plane, parts_all = 0, cut_all = 0;
  for (int p = 0; p < Mb; ++p) {
    if (p < m) {
      q += part_s[p][0];
      rho += part_s[p][1];
    }
    parts_all += part_s[p][0];
    cut_all += part_s[p][1];
  }
  if (threadIdx.x == 0) {
    sched[kSchedNParts] = parts_all;
    sched[kSchedSplitT] = T;
    sched[kSchedNCutRows] = cut_all;
    for (int x = 3; x < kSchedPartBase; ++x) sched[x] = 0;
  }
  if (!live) return;
  // list entry number n of this row, from the masks (the same value the fill above stored)
  auto entry_at = [&](int n) {
#pragma unroll
    for (int ch = 0; ch < kTinyMaxChunks; ++ch) {
      uint64_t x = nz[ch];
      const int cnt = __popcll(x);
      if (n < cnt) {
        for (int t = 0; t < n; ++t) x &= x - 1;
        const int b = ctz64(x);
        return (int)((uint32_t)(64 * ch + b) | (((full[ch] >> b) & 1ull) ? 0x80000000u : 0u));
      }
      n -= cnt;
    }
    return -1;
  };
  if (np > 0) {
    const int chunk = (c + np - 1) / np;
    for (int k = 0; k < np; ++k) {
      int32_t* rec = sched + kSchedPartBase + (int64_t)kSchedPartInts * (q + k);
      rec[0] = m * nbr + i;
      rec[1] = start + k * chunk;
      rec[2] = min(chunk, c - k * chunk);
      rec[3] = k;
      rec[4] = np;
      rec[5] = q;
      rec[6] = rho;
      rec[7] = entry_at(k * chunk);
    }
  }
  const int rank = launch_rank(len_s[m], gmax_s[m], nbr, gsz, i);
  reinterpret_cast<int4*>(sched + sched_order_base(Mb, nbr))[(int64_t)m * nbr + rank] = make_int4(i, start, c, entry_at(0));
}

// Whole sparse index (row_ptr, col_idx and, if asked for, the schedule), and if asked for the run index as well,
// in ONE launch of one work-group, for class matrices of at most kSmallPairs (row, 64-column chunk) pairs -- e.g. 4 planes of a 4096 x 4096 mask in 128 x 64
// tiles.  At this size the four launches of the general path cost far more than the work itself.  Pair p = (row r,
// chunk ch) with p = r*CH + ch is owned by slot p % 16 of wave p / 16; lists are row-major and ascending, so the
// position of a pair's first entry in its plane's list is the exclusive prefix sum of the pairs' popcounts.
constexpr int kSmallWaves = 16, kSmallSlots = 16, kSmallPairs = kSmallWaves * kSmallSlots;

__global__ __launch_bounds__(kSmallWaves * 64) void small_index_kernel(const uint8_t* __restrict__ cls, int Mb, int nbr,
                                                                       int nbc, int32_t* __restrict__ row_ptr,
                                                                       uint32_t* col_idx, int32_t* __restrict__ sched,
                                                                       int32_t* __restrict__ offset,
                                                                       int32_t* __restrict__ total_ones,
                                                                       int32_t* __restrict__ nz_lo,
                                                                       int32_t* __restrict__ nz_hi,
                                                                       int32_t* __restrict__ nz_cnt) {
  using namespace bbm;
  __shared__ int pc[kSmallPairs];     // non-zero blocks of a pair
  __shared__ int pos[kSmallPairs];    // position of the pair's first entry in the plane's list
  __shared__ int len_s[kSmallPairs];  // list length of a row
  __shared__ int gmax_s[kSmallPairs]; // longest list of a launch-order group (groups never span planes)
  __shared__ int np_s[kSmallPairs];   // parts of a row (0 = not cut)
  __shared__ int tot_s[4];            // list entries, non-empty rows, parts, cut rows
  __shared__ int gpre_s[kSmallPairs], wsum_s[kSmallPairs / 64];
  __shared__ uint64_t full_s[kSmallPairs], nz_s[kSmallPairs];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: pair -> (row, chunk) arithmetic stays off the vector ALU
  const int CH = (nbc + 63) / 64, PP = nbr * CH, npairs = Mb * PP, nrows = Mb * nbr;
  const int64_t plane_entries = (int64_t)nbr * nbc;
  if (tid < 4) tot_s[tid] = 0;

  // (row, chunk, plane) of the wave's first pair by division, of the following ones by counting (integer division is
  // dozens of instructions)
  const int r_first = wave * kSmallSlots / CH, ch_first = wave * kSmallSlots - r_first * CH, m_first = r_first / nbr;
  uint8_t v[kSmallSlots];
  uint64_t nz[kSmallSlots];
  {
    int r = r_first, ch = ch_first;
#pragma unroll
    for (int k = 0; k < kSmallSlots; ++k) {
      const int p = wave * kSmallSlots + k, col = ch * 64 + lane;
      v[k] = (p < npairs && col < nbc) ? cls[(int64_t)r * nbc + col] : (uint8_t)0;
      if (++ch == CH) {
        ch = 0;
        ++r;
      }
    }
  }
#pragma unroll
  for (int k = 0; k < kSmallSlots; ++k) {
    const int p = wave * kSmallSlots + k;
    nz[k] = __ballot(v[k] != BBM_BLOCK_EMPTY);
    const uint64_t full = __ballot(v[k] == BBM_BLOCK_FULL);
    if (lane == 0 && p < npairs) {
      pc[p] = __popcll(nz[k]);
      nz_s[p] = nz[k];
      full_s[p] = full;
    }
  }
  __syncthreads();
  // exclusive prefix sums of pc over all pairs (the first four waves scan 64 pairs each), then made plane-relative
  if (wave < kSmallPairs / 64) {
    const int x = tid < npairs ? pc[tid] : 0;
    int incl = x;
    for (int d = 1; d < 64; d <<= 1) {
      const int y = __shfl_up(incl, d);
      if (lane >= d) incl += y;
    }
    if (lane == 63) wsum_s[wave] = incl;
    gpre_s[tid] = incl - x;
  }
  __syncthreads();
  if (tid < npairs) {
    const int q0 = tid / PP * PP;  // first pair of this pair's plane
    int own = 0, first = 0;
    for (int w = 0; w < kSmallPairs / 64; ++w) {
      own += w < wave ? wsum_s[w] : 0;
      first += w < (q0 >> 6) ? wsum_s[w] : 0;
    }
    pos[tid] = gpre_s[tid] + own - (gpre_s[q0] + first);
  }
  __syncthreads();
  int c = 0, start = 0;  // list length and list position of row `tid`
  if (tid < nrows) {
    const int m = tid / nbr, i = tid - m * nbr, p0 = tid * CH;
    start = pos[p0];
    const int end = (i == nbr - 1) ? pos[p0 + CH - 1] + pc[p0 + CH - 1] : pos[p0 + CH];
    c = end - start;
    row_ptr[(int64_t)m * (nbr + 1) + i] = start;
    if (i == nbr - 1) row_ptr[(int64_t)m * (nbr + 1) + nbr] = end;
    len_s[tid] = c;
    if (c > 0) {
      atomicAdd(&tot_s[0], c);
      atomicAdd(&tot_s[1], 1);
    }
  }
  {
    int r = r_first, ch = ch_first, m = m_first;
#pragma unroll
    for (int k = 0; k < kSmallSlots; ++k) {
      const int p = wave * kSmallSlots + k;
      if (p < npairs && ((nz[k] >> lane) & 1ull))
        col_idx[(int64_t)m * plane_entries + pos[p] + __popcll(nz[k] & ((1ull << lane) - 1ull))] =
            (uint32_t)(ch * 64 + lane) | (v[k] == BBM_BLOCK_FULL ? 0x80000000u : 0u);
      if (++ch == CH) {
        ch = 0;
        if (++r == (m + 1) * nbr) ++m;
      }
    }
  }
  if (offset && tid < nrows) {  // run index: this thread walks the chunks of its row
    RunScan rs;
    for (int ch = 0; ch < CH; ++ch) rs.feed(full_s[tid * CH + ch], nz_s[tid * CH + ch], 64 * ch);
    rs.finish();
    offset[tid] = rs.best_start;
    total_ones[tid] = rs.best_len;
    nz_lo[tid] = rs.lo;
    nz_hi[tid] = rs.hi;
    nz_cnt[tid] = rs.cnt;
  }
  if (!sched) return;
  __syncthreads();  // totals complete
  // list entry number n of row r, from the chunk masks (the same value the fill above stores)
  auto entry_at = [&](int r, int n) {
    for (int ch = 0; ch < CH; ++ch) {
      uint64_t x = nz_s[r * CH + ch];
      const int cnt = __popcll(x);
      if (n < cnt) {
        for (int t = 0; t < n; ++t) x &= x - 1;
        const int bit = ctz64(x);
        return (int)((uint32_t)(64 * ch + bit) | (((full_s[r * CH + ch] >> bit) & 1ull) ? 0x80000000u : 0u));
      }
      n -= cnt;
    }
    return -1;
  };

  // ---- schedule (same definition as sched_kernel; everything sits in LDS here)
  const int total = tot_s[0], nonempty = tot_s[1];
  const int mean = nonempty > 0 ? (total + nonempty - 1) / nonempty : 0;
  const int T = max(kSchedMinSplit, 2 * mean);
  const int np = (tid < nrows && c > T) ? (c + T - 1) / T : 0;
  if (tid < nrows) np_s[tid] = np;
  if (np > 0) {
    atomicAdd(&tot_s[2], np);
    atomicAdd(&tot_s[3], 1);
  }
  const int gsz = launch_group_rows(T), ngp = (nbr + gsz - 1) / gsz;  // launch-order groups: rows each, groups per plane
  if (tid < Mb * ngp) {
    const int m = tid / ngp, g = tid - m * ngp;
    int t = 0;
    for (int j = g * gsz; j < min(nbr, (g + 1) * gsz); ++j) t = max(t, len_s[m * nbr + j]);
    gmax_s[tid] = t;
  }
  __syncthreads();
  if (tid == 0) {
    sched[kSchedNParts] = tot_s[2];
    sched[kSchedSplitT] = T;
    sched[kSchedNCutRows] = tot_s[3];
    for (int x = 3; x < kSchedPartBase; ++x) sched[x] = 0;
  }
  if (tid < nrows) {
    const int m = tid / nbr, i = tid - m * nbr;
    if (np > 0) {
      int q = 0, rho = 0;
      for (int r = 0; r < tid; ++r) {
        q += np_s[r];
        rho += np_s[r] > 0;
      }
      const int chunk = (c + np - 1) / np;
      for (int k = 0; k < np; ++k) {
        int32_t* rec = sched + kSchedPartBase + (int64_t)kSchedPartInts * (q + k);
        rec[0] = tid;
        rec[1] = start + k * chunk;
        rec[2] = min(chunk, c - k * chunk);
        rec[3] = k;
        rec[4] = np;
        rec[5] = q;
        rec[6] = rho;
        rec[7] = entry_at(tid, k * chunk);
      }
    }
    const int rank = launch_rank(len_s + m * nbr, gmax_s + m * ngp, nbr, gsz, i);
    reinterpret_cast<int4*>(sched + sched_order_base(Mb, nbr))[(int64_t)m * nbr + rank] =
        make_int4(i, start, c, entry_at(tid, 0));
  }
}

}  // namespace

namespace {

int check_runs_args(const char* fn, const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, const int32_t* offset,
                    const int32_t* total_ones, const int32_t* nz_lo, const int32_t* nz_hi, const int32_t* nz_cnt) {
  using namespace bbm;
  if (!blk_class || !offset || !total_ones || !nz_lo || !nz_hi || !nz_cnt) return fail(BBM_EINVAL, "%s: NULL pointer argument", fn);
  if (Mb < 1 || nbr < 1 || nbc < 1)
    return fail(BBM_EINVAL, "%s: Mb=%lld, nbr=%lld, nbc=%lld must be >= 1", fn, (long long)Mb, (long long)nbr, (long long)nbc);
  if (nbc > (1ll << 30) || Mb * nbr > (1ll << 31) * kWavesPerWG - 1) return fail(BBM_EUNSUPPORTED, "%s: index too large", fn);
  return BBM_OK;
}

int check_list_args(const char* fn, const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, const int32_t* row_ptr,
                    const uint32_t* col_idx, const int32_t* sched) {
  using namespace bbm;
  if (!blk_class || !row_ptr || !col_idx) return fail(BBM_EINVAL, "%s: NULL pointer argument", fn);
  if (Mb < 1 || nbr < 1 || nbc < 1)
    return fail(BBM_EINVAL, "%s: Mb=%lld, nbr=%lld, nbc=%lld must be >= 1", fn, (long long)Mb, (long long)nbr, (long long)nbc);
  if (nbr * nbc >= (1ll << 31) || Mb * nbr >= (1ll << 24))
    return fail(BBM_EUNSUPPORTED, "%s: needs nbr*nbc=%lld < 2^31 and Mb*nbr=%lld < 2^24", fn, (long long)(nbr * nbc), (long long)(Mb * nbr));
  if (sched && !aligned(sched, 32)) return fail(BBM_EINVAL, "%s: sched must be 32-byte aligned", fn);
  return BBM_OK;
}

int launch_runs(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, int32_t* offset, int32_t* total_ones,
                int32_t* nz_lo, int32_t* nz_hi, int32_t* nz_cnt, int32_t* row_ptr_counts, hipStream_t s) {
  const int64_t rows = Mb * nbr;
  runs_kernel<<<(unsigned)bbm::ceil_div(rows, kWavesPerWG), kWavesPerWG * 64, 0, s>>>(blk_class, rows, nbc, offset, total_ones,
                                                                                    nz_lo, nz_hi, nz_cnt, row_ptr_counts, nbr);
  return bbm::launch_status("bbm_build_runs");
}

bool is_small(int64_t Mb, int64_t nbr, int64_t nbc) { return Mb * nbr * bbm::ceil_div(nbc, (int64_t)64) <= kSmallPairs; }
bool is_tiny(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc) {
  return Mb <= kTinyMaxPlanes && nbr <= kTinyMaxRows && nbc <= 64 * kTinyMaxChunks && nbc % 16 == 0 && bbm::aligned(blk_class, 16);
}

// One-launch paths for small class matrices; returns false if neither applies.
bool launch_one_kernel(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, int32_t* row_ptr, uint32_t* col_idx,
                       int32_t* sched, int32_t* offset, int32_t* total_ones, int32_t* nz_lo, int32_t* nz_hi, int32_t* nz_cnt,
                       hipStream_t s) {
  if (is_tiny(blk_class, Mb, nbr, nbc)) {
    tiny_index_kernel<<<1, (unsigned)Mb * 64, 0, s>>>(blk_class, (int)Mb, (int)nbr, (int)nbc, row_ptr, col_idx, sched, offset,
                                                       total_ones, nz_lo, nz_hi, nz_cnt);
    return true;
  }
  if (is_small(Mb, nbr, nbc)) {
    small_index_kernel<<<1, kSmallWaves * 64, 0, s>>>(blk_class, (int)Mb, (int)nbr, (int)nbc, row_ptr, col_idx, sched, offset,
                                                      total_ones, nz_lo, nz_hi, nz_cnt);
    return true;
  }
  return false;
}

// `counts`: per-row list lengths [Mb][nbr] already on the stream (the runs kernel's nz_cnt), or NULL.  With them the
// count launch is not needed, nor -- up to kScanInFillRows block rows per plane -- the scan launch.
constexpr int64_t kScanInFillRows = 1024;
int launch_list(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, int32_t* row_ptr, uint32_t* col_idx,
                int32_t* sched, const int32_t* counts, bool counts_in_row_ptr, hipStream_t s) {
  using namespace bbm;
  if (!counts && launch_one_kernel(blk_class, Mb, nbr, nbc, row_ptr, col_idx, sched, nullptr, nullptr, nullptr, nullptr, nullptr, s))
    return launch_status("bbm_build_sparse_index(one launch)");
  const unsigned grid = (unsigned)ceil_div(Mb * nbr, kWavesPerWG);
  int rc = BBM_OK;
  const bool scan_in_fill = counts && nbr <= kScanInFillRows;
  if (!scan_in_fill) {
    if (!counts_in_row_ptr) {
      list_count_kernel<<<grid, kWavesPerWG * 64, 0, s>>>(blk_class, Mb, nbr, nbc, row_ptr);
      rc = launch_status("bbm_build_sparse_index(count)");
      if (rc) return rc;
    }
    list_scan_kernel<<<(unsigned)Mb, 64, 0, s>>>(nbr, row_ptr);
    rc = launch_status("bbm_build_sparse_index(scan)");
    if (rc) return rc;
  }
  if (scan_in_fill && sched && Mb * nbr <= kFuseSchedRows) {  // list and schedule in one launch
    list_fill_sched_kernel<<<grid, kWavesPerWG * 64, 0, s>>>(blk_class, (int)Mb, (int)nbr, (int)nbc, row_ptr, counts, col_idx, sched);
    return launch_status("bbm_build_sparse_index(fill and schedule)");
  }
  list_fill_kernel<<<grid, kWavesPerWG * 64, 0, s>>>(blk_class, Mb, nbr, nbc, row_ptr, scan_in_fill ? counts : nullptr, col_idx);
  rc = launch_status("bbm_build_sparse_index(fill)");
  if (rc || !sched) return rc;
  sched_kernel<<<(unsigned)(1 + Mb), kSchedThreads, 0, s>>>(row_ptr, col_idx, (int)Mb, (int)nbr, nbr * nbc, sched);
  return launch_status("bbm_build_sparse_index(schedule)");
}

}  // namespace

extern "C" __attribute__((visibility("default"))) int bbm_build_runs(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, int32_t* offset,
                              int32_t* total_ones, int32_t* nz_lo, int32_t* nz_hi, int32_t* nz_cnt, void* stream) {
  bbm::clear_error();
  const int rc = check_runs_args("bbm_build_runs", blk_class, Mb, nbr, nbc, offset, total_ones, nz_lo, nz_hi, nz_cnt);
  if (rc) return rc;
  return launch_runs(blk_class, Mb, nbr, nbc, offset, total_ones, nz_lo, nz_hi, nz_cnt, nullptr, static_cast<hipStream_t>(stream));
}

extern "C" __attribute__((visibility("default"))) size_t bbm_sched_bytes(int64_t Mb, int64_t nbr) {
  if (Mb < 1 || nbr < 1) return 0;
  return (size_t)bbm::sched_ints(Mb, nbr) * sizeof(int32_t);
}

extern "C" __attribute__((visibility("default"))) int bbm_build_sparse_index(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc,
                                      int32_t* row_ptr, uint32_t* col_idx, int32_t* sched, void* stream) {
  bbm::clear_error();
  const int rc = check_list_args("bbm_build_sparse_index", blk_class, Mb, nbr, nbc, row_ptr, col_idx, sched);
  if (rc) return rc;
  return launch_list(blk_class, Mb, nbr, nbc, row_ptr, col_idx, sched, nullptr, false, static_cast<hipStream_t>(stream));
}

extern "C" __attribute__((visibility("default"))) int bbm_build_index(const uint8_t* blk_class, int64_t Mb, int64_t nbr, int64_t nbc, int32_t* offset,
                               int32_t* total_ones, int32_t* nz_lo, int32_t* nz_hi, int32_t* nz_cnt, int32_t* row_ptr,
                               uint32_t* col_idx, int32_t* sched, void* stream) {
  using namespace bbm;
  clear_error();
  int rc = check_runs_args("bbm_build_index", blk_class, Mb, nbr, nbc, offset, total_ones, nz_lo, nz_hi, nz_cnt);
  if (rc) return rc;
  rc = check_list_args("bbm_build_index", blk_class, Mb, nbr, nbc, row_ptr, col_idx, sched);
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (launch_one_kernel(blk_class, Mb, nbr, nbc, row_ptr, col_idx, sched, offset, total_ones, nz_lo, nz_hi, nz_cnt, s))
    return launch_status("bbm_build_index(one launch)");
  // the runs kernel's counts are pass 1 of the list: in nz_cnt for the fill kernel, and in row_ptr where a scan launch follows
  const bool scan_launch = nbr > kScanInFillRows;
  rc = launch_runs(blk_class, Mb, nbr, nbc, offset, total_ones, nz_lo, nz_hi, nz_cnt, scan_launch ? row_ptr : nullptr, s);
  if (rc) return rc;
  return launch_list(blk_class, Mb, nbr, nbc, row_ptr, col_idx, sched, nz_cnt, scan_launch, s);
}
