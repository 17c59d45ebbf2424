// Stage 2: fused masked attention forward that visits only non-zero key/value tiles (paper Sec. 3 "Flash
// Attention", Sec. 4 "Binary Block Masking" / "Dense Binary Block Masking").
//
// Work decomposition.  One work-group owns one block row (Br = 32*NW query rows) of one (batch, head); each
// of its NW wavefronts owns 32 query rows.  Key/value tiles are Bc = 64 keys wide.  The kernel computes the
// TRANSPOSED products so that one lane owns one query row:
//     S^T[key][q]  = K_tile[key][:] . Q[q][:]        (A operand = K from LDS, B operand = Q in registers)
//     O^T[dcol][q] += V_tile^T[dcol][key] . P^T[key][q]  (A operand = V via transposing LDS reads, B = P)
// With the 32x32x16 bf16 MFMA the accumulator of lane l holds column q = l%32 and rows
// 8*(v/4) + 4*(l/32) + v%4, v = 0..15.  So a lane and its partner l^32 together hold all scores of one query
// row: the row maximum needs one cross-lane exchange, the rescale factor and the row sum stay in-lane, and
// the S^T accumulators are -- after rounding to bf16 -- directly the B operand of the second product (the key
// order inside a 16-key MFMA step is a fixed permutation, matched by the addresses of the V reads).
// The element mask of a 32x64 score slab is one 64-bit word per query row (word-column-major packed mask),
// tested with compile-time bit positions.
#include "bbm_internal.h"

#include <algorithm>
#include <mutex>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBc = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazy = 8.0f;  // log2 headroom before the running maximum is moved

struct AttnParams {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  __bf16* o;
  float* lse;
  const uint64_t* packed;  // [Mb][W][N]
  const uint8_t* bin_blk_mat;
  const int32_t* offset;
  const int32_t* total_ones;
  const int32_t* nz_lo;
  const int32_t* nz_hi;
  const int32_t* row_ptr;
  const uint32_t* col_idx;
  int64_t N;   // queries per head
  int64_t Nk;  // keys per head (= N for self-attention over one sequence)
  int32_t H, Mb, nbr, nbc, W;
  int32_t total_wgs;
  int32_t mode;
  float qscale;       // factor applied to Q before it is rounded to bf16 (see `rmul`)
  float rmul;         // factor applied to the first product's result inside the exponential (EXACT instances), else 1
  // LIST mode: schedule (read-only), work-queue state and partial results of cut rows (in the caller's workspace)
  const int32_t* sched;
  int32_t* queue;     // [0] part items handed out, [1] leading work-groups done, [8 + rho*hbp + hb] finished parts of
                      // cut row rho; all zero between calls (each call puts back the zeros it disturbed)
  float* partials;    // [(cut part)*hbp + hb][regs + 2][threads]
  int32_t hbp;        // (batch, head) pairs per mask plane: B*H if Mb == 1, else H
  int32_t n_extra;    // leading work-groups that serve the queue of cut-row parts (LIST mode)
  int32_t G;          // (batch, head) planes whose block rows are interleaved in launch order
  int32_t split;      // parts per block row when the launch is too small to fill the chip (LIST mode), else 1
  int32_t part_cap;   // records of `partials` the workspace holds; a schedule whose parts need more is not followed
};

__device__ __forceinline__ float partner_max(float x) {
  // lanes l and l^32 exchange: swap(x, x) gives {x[l%32], x[l%32 + 32]} in some order on every lane
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float partner_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

constexpr int kWin = 1024;               // tiles per schedule window (block columns, or list entries)
constexpr uint32_t kNoTile = 0xffffffffu;  // sentinel after the last entry of a window
constexpr uint32_t kZeroWord = 0x40000000u;  // entry flag: the tile's mask words are all zero and are not in memory

// Builds, in LDS, the ascending list of tiles one block row visits inside one schedule window; entry =
// block column | (1 << 31 if the element mask can be skipped there).  Returns the number of entries (uniform).
// `win` counts windows of kWin block columns.  (BITMAP, RUNS and DENSE_BASELINE; LIST mode copies its list instead.)
// [clo, chi): the block columns this work-group is responsible for (all of them unless the block row is computed in
// parts).
template <int NW>
__device__ __forceinline__ int build_window(const AttnParams& P, int m, int i, int win, uint32_t* tiles_s, int* cnt_s, int clo, int chi) {
  constexpr int NT = NW * 64;
  constexpr int CH = kWin / 64;  // 64-column chunks per window
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t r = (int64_t)m * P.nbr + i;
  int count;
  if (P.mode == BBM_MODE_DENSE_BASELINE) {
    const int j0 = clo + win * kWin;
    count = min(kWin, chi - j0);
    // an empty block's packed words are never written by the block reduction: flag it, the mask word is then 0
    const uint8_t* row = P.bin_blk_mat + r * P.nbc;
    for (int t = tid; t < count; t += NT) tiles_s[t] = (uint32_t)(j0 + t) | (row[j0 + t] == 0 ? kZeroWord : 0u);
  } else {
    int lo = clo, hi = chi, run_lo = 0, run_hi = 0;
    if (P.mode == BBM_MODE_RUNS) {
      lo = max(clo, P.nz_lo[r]);
      hi = min(chi, P.nz_hi[r]);
      run_lo = P.offset[r];
      run_hi = run_lo + P.total_ones[r];
    }
    const int j0 = (lo & ~63) + win * kWin;
    const uint8_t* row = P.bin_blk_mat + r * P.nbc;
    uint64_t nz[(CH + NW - 1) / NW];
#pragma unroll
    for (int n = 0; n < (CH + NW - 1) / NW; ++n) {
      const int ch = wave + n * NW;
      const int j = j0 + 64 * ch + lane;
      const uint8_t v = (ch < CH && j >= lo && j < hi) ? row[j] : (uint8_t)0;
      nz[n] = __ballot(v != 0);
      if (ch < CH && lane == 0) cnt_s[ch] = __popcll(nz[n]);
    }
    __syncthreads();
    int total = 0, before = 0;
    for (int ch = 0; ch < CH; ++ch) {
      const int cn = cnt_s[ch];
      total += cn;
    }
    count = total;
#pragma unroll
    for (int n = 0; n < (CH + NW - 1) / NW; ++n) {
      const int ch = wave + n * NW;
      if (ch < CH) {
        before = 0;
        for (int c2 = 0; c2 < ch; ++c2) before += cnt_s[c2];
        if ((nz[n] >> lane) & 1ull) {
          const int j = j0 + 64 * ch + lane;
          const bool in_run = (P.mode == BBM_MODE_RUNS) && j >= run_lo && j < run_hi;
          tiles_s[before + __popcll(nz[n] & ((1ull << lane) - 1ull))] = (uint32_t)j | (in_run ? 0x80000000u : 0u);
        }
      }
    }
  }
  count = __builtin_amdgcn_readfirstlane(count);
  if (tid < 3) tiles_s[count + tid] = kNoTile;
  __syncthreads();
  return count;
}

// Number of schedule windows of the block columns [clo, chi) of one block row (uniform).
__device__ __forceinline__ int num_windows(const AttnParams& P, int m, int i, int clo, int chi) {
  int lo = clo, hi = chi;
  if (P.mode == BBM_MODE_RUNS) {
    const int64_t r = (int64_t)m * P.nbr + i;
    lo = max(clo, P.nz_lo[r]);
    hi = min(chi, P.nz_hi[r]);
  }
  if (hi <= lo) return 0;
  if (P.mode != BBM_MODE_DENSE_BASELINE) lo &= ~63;
  return (hi - lo + kWin - 1) / kWin;
}

template <int V>
struct IntC {
  static constexpr int value = V;
};

// One work-group per (block row, batch, head), tiles from build_window.  SCHED = 2 (LIST mode on a launch too small to
// fill the chip): every block row is computed in P.split equal parts by as many work-groups, merged like cut rows.
// With SCHED = 1 (LIST mode) the first
// P.n_extra work-groups, before turning to their own block row, take the parts of the block rows which the split
// schedule cut from a queue; the work-group that completes a row's last part merges the parts in part order and
// writes the row, and the row's own work-group skips it.
//
// The softmax needs exp2(c * <q, k> - m) with c = softmax_scale * log2(e).  EXACT = false: Q is multiplied by c and
// rounded to bf16, so the first product delivers the exponent directly (no per-element multiplication; the rounding
// moves a score by up to 2^-9 * c * sum |q_d k_d|, harmless up to the usual scale 1/sqrt(d)).  EXACT = true (sharper
// scales): c = 2^k * r with r in [1, 2); Q is multiplied by 2^k, which is exact in bf16, and r multiplies the
// accumulator inside the exponential; running maxima are then kept in units of 1/r.
template <int D, int NW, int SCHED, bool EXACT>
__global__ __launch_bounds__(NW * 64) void attn_fwd_kernel(const AttnParams P) {
  constexpr int NT = NW * 64;
  constexpr int BR = NW * 32;
  // LDS tile layout ("blocks"): one asynchronous copy instruction of a wave fills one 1 KiB block with RPB rows
  // that lie NBLK rows apart: row r sits in block r % NBLK at slot r / NBLK.  Blocks are padded (K by 16 bytes, V
  // by 64) so that the 16 consecutive rows a 16-byte K read touches, and the 4 consecutive rows a transposing V
  // read touches, start in different banks.  Every read address is one per-lane register plus a constant.
  constexpr int RC = D / 8;                    // 16-byte chunks per row
  constexpr int RPB = 64 / RC;                 // rows per 1 KiB block
  constexpr int NBLK = kBc / RPB;              // blocks per tile = copy instructions per tile
  constexpr int LPW = NBLK / NW;               // copy instructions per wave and tile
  static_assert(NBLK % NW == 0, "tile must split evenly over the waves");
  constexpr int KBLK = 512 + 8;                // K block stride in elements (1 KiB + 16 B)
  constexpr int VBLK = 512 + 32;               // V block stride in elements (1 KiB + 64 B)
  constexpr int KS = D / 16;                   // MFMA k-steps of the first product
  constexpr int DB = D / 32;                   // 32-wide output-column blocks of the second product
  constexpr int REGS = DB * 16;                // fp32 accumulator registers per lane
  static_assert(2 * 32 * D <= NBLK * KBLK && NW <= 8, "two 32 x D output slabs must fit in each tile buffer");

  // separate arrays per buffer so the compiler can tell an asynchronous copy into one from reads of the other
  __shared__ __attribute__((aligned(16))) __bf16 k_s0[NBLK * KBLK];
  __shared__ __attribute__((aligned(16))) __bf16 k_s1[NBLK * KBLK];
  __shared__ __attribute__((aligned(16))) __bf16 v_s0[NBLK * VBLK];
  __shared__ __attribute__((aligned(16))) __bf16 v_s1[NBLK * VBLK];
  __shared__ uint32_t tiles_s[kWin + 4];
  __shared__ int cnt_s[kWin / 64];
  __shared__ int item_s[2];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction: keep it in a scalar register
  const int lq = lane & 31, hh = lane >> 5;
  const int64_t N = P.N, Nk = P.Nk;
  const float c = P.qscale;
  const float rr = EXACT ? P.rmul : 1.0f;
  auto ex2 = [&](float x) { return __builtin_amdgcn_exp2f(EXACT ? rr * x : x); };

  // ---- per-item state (SCHED = false: exactly one item, derived from blockIdx)
  int m, i, bh;
  const __bf16* __restrict__ Kg;
  const __bf16* __restrict__ Vg;
  int64_t head_off, qrow;
  bool q_ok;
  const uint64_t* __restrict__ mrow;
  bf16x8 qf[KS];
  f32x16 oacc[DB];
  // m_run: reference maximum of the row in exponent units (score * scale * log2 e; -inf before the first visible key);
  // s_init: its negative (0 while m_run = -inf), replicated, as the start value of the score accumulators
  float m_run, l_run;
  f32x16 s_init;

  // Q through LDS needs a 32 x D staging slab per wave in the two buffers of parity 1 (two slabs each)
  constexpr bool Q_VIA_LDS = NW <= 4;
  bool q_pending = false;
  const int g_row = lane / RC, g_chunk = lane % RC;  // row and 16-byte chunk this lane moves in a 1 KiB copy
  auto q_stage = [&]() { return (wave / 2 == 0 ? k_s1 : v_s1) + (wave % 2) * 32 * D; };
  auto begin_item = [&]() {
    head_off = (int64_t)bh * N * D;
    Kg = P.k + (int64_t)bh * Nk * D;
    Vg = P.v + (int64_t)bh * Nk * D;
    qrow = (int64_t)i * BR + wave * 32 + lq;
    q_ok = qrow < N;
    // packed mask words of this lane's query row (rows past N borrow row 0: their results are never stored)
    mrow = P.packed + (int64_t)m * P.W * N + (q_ok ? qrow : 0);
    if constexpr (Q_VIA_LDS) {
      // The wave's 32 x D slab of Q is one contiguous piece of memory: copy it asynchronously, 1 KiB per instruction,
      // into this wave's staging slab (tile buffer 1, idle until the second tile is requested) and pick the MFMA
      // fragments up from there in fetch_q.  Chunk j of row r lands at chunk position j ^ (r % RC) of row r.  Rows
      // past N re-read row N-1 (their results are never stored).
      const int64_t row0 = (int64_t)i * BR + wave * 32;
      const char* slab = reinterpret_cast<const char*>(P.q + head_off + row0 * D);
      const int last = (int)min<int64_t>(31, N - 1 - row0);  // >= 0 for every wave that owns a real row
      __bf16* const stage = q_stage();
#pragma unroll
      for (int n = 0; n < 32 / RPB; ++n) {
        const int r = min(n * RPB + g_row, last);
        const uint32_t off = (uint32_t)(r * D + ((g_chunk ^ (r % RC)) * 8)) * 2u;
        if (last >= 0)
          __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(slab + off),
                                           (void __attribute__((address_space(3)))*)(stage + n * 512), 16, 0, 0);
      }
      q_pending = true;
    } else {
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        if (q_ok)
          qf[t] = *reinterpret_cast<const bf16x8*>(P.q + head_off + qrow * D + 16 * t + 8 * hh);
        else
          for (int e = 0; e < 8; ++e) qf[t][e] = (__bf16)0.0f;
        for (int e = 0; e < 8; ++e) qf[t][e] = (__bf16)((float)qf[t][e] * c);
      }
    }
#pragma unroll
    for (int db = 0; db < DB; ++db)
      for (int e = 0; e < 16; ++e) oacc[db][e] = 0.0f;
    m_run = -INFINITY;
    l_run = 0.0f;
    for (int e = 0; e < 16; ++e) s_init[e] = 0.0f;
  };

  // Asynchronous global -> LDS copy (no registers in between).  One instruction moves 1 KiB per wave: lane l lands at
  // LDS base + 16*l, i.e. slot l / RC, chunk l % RC of the block, so it fetches row (block + NBLK * slot).
  // Addresses are (uniform 64-bit tile base) + (32-bit per-lane byte offset): one register per lane, not a pair per copy.
  const uint32_t g_off = (uint32_t)(g_row * NBLK * D + g_chunk * 8) * 2u;
  auto load_tile_async = [&](const __bf16* __restrict__ src, int jt, __bf16* dst, int blk_stride) {
    const int64_t key0 = (int64_t)jt * kBc;
    const char* tile = reinterpret_cast<const char*>(src + key0 * D);
    if (key0 + kBc <= Nk) {
#pragma unroll
      for (int n = 0; n < LPW; ++n) {
        const int q = n * NW + wave;  // block filled by this instruction
        __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(tile + q * D * 2 + g_off),
                                         (void __attribute__((address_space(3)))*)(dst + q * blk_stride), 16, 0, 0);
      }
    } else {
      // Last tile of a ragged key count Nk.  Rows past Nk re-read row Nk-1: such keys sit in a tile that is never "full", the
      // element mask gives them probability exactly 0, and a finite duplicate row then adds nothing.
      const int last = (int)(Nk - 1 - key0);  // last real row of the tile
#pragma unroll
      for (int n = 0; n < LPW; ++n) {
        const int q = n * NW + wave;
        const uint32_t off = (uint32_t)(min(q + g_row * NBLK, last) * D + g_chunk * 8) * 2u;
        __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(tile + off),
                                         (void __attribute__((address_space(3)))*)(dst + q * blk_stride), 16, 0, 0);
      }
    }
  };

  // K fragment of MFMA k-step t, key block kb: row 32*kb + lq, chunk 2t + hh.
  const int kaddr = (lq % NBLK) * KBLK + (lq / NBLK) * D + hh * 8;
  // S^T = K Q^T for the 64 keys of one LDS tile x this wave's 32 queries
  // The K fragments go through a ring of kRing register sets, each requested kRing matrix instructions before the one
  // that consumes it; the scheduling hints pin that order (left to itself the compiler issues every LDS read right
  // before its MFMA, which then waits out the LDS latency: d=128 dense -1.2 %, tree -3 %; a ring of 8 costs the d=64
  // kernel its third wave per SIMD, the same treatment of the V fragments of the second product gains nothing).
  auto qk = [&](const __bf16* ks, f32x16 (&s)[2]) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) s[kb] = s_init;
    constexpr int NF = 2 * KS, kRing = 4;
    auto frag = [&](int n) {  // fragment n: MFMA k-step n / 2, key block n % 2
      return *reinterpret_cast<const bf16x8*>(ks + kaddr + (n & 1) * (32 / NBLK) * D + (n >> 1) * 16);
    };
    bf16x8 ring[kRing];
#pragma unroll
    for (int n = 0; n < kRing; ++n) ring[n] = frag(n);
#pragma unroll
    for (int n = 0; n < NF; ++n) {
      const bf16x8 kf = ring[n % kRing];
      if (n + kRing < NF) ring[n % kRing] = frag(n + kRing);
      s[n & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[n >> 1], s[n & 1], 0, 0, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, kRing, 0);  // kRing LDS reads, then (MFMA, LDS read) pairs, then the last MFMAs
#pragma unroll
    for (int n = 0; n < NF - kRing; ++n) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, kRing, 0);
  };

  // V fragment (transposing read) of 16-key step u, half a, column block db: the lane addresses row
  // vr = 16u + 8a + 4hh + y (y = (lane%16)/4), 16-byte chunk 4db + 2g + x (g = (lane/16)%2, x = (lane%4)/2),
  // elements 4*(lane%2).. of it, and receives keys 16u + 8a + 4hh + 0..3 of column 32db + lane%32 -- the key
  // order of the bf16 probabilities taken straight from the S^T accumulators.
  const int vy = (lane & 15) >> 2, vg = (lane >> 4) & 1, vx = (lane & 3) >> 1;
  const int vaddr = (4 * hh + vy) * VBLK + (2 * vg + vx) * 8 + 4 * (lane & 1);
  auto v_frag = [&](const __bf16* vs, int u, int db) {
    s16x4 part[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      // row 16u + 8a + (4hh + y): block (row % NBLK), slot (row / NBLK)
      const int off = D == 64 ? (2 * u + a) * D + db * 32 : 8 * a * VBLK + u * D + db * 32;
      part[a] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vs + vaddr + off));
    }
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7));
  };

  auto tile_of = [](uint32_t e) { return e == kNoTile ? -1 : (int)(e & 0x3fffffffu); };
  const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};

  // One tile: S^T = K Q^T, mask, online softmax and O^T += V^T P^T for tile e0 whose K and V sit in buffer PB; the
  // asynchronous copies of the next tile into the other buffer are started first.
  uint32_t e0, e1;
  uint64_t mw_nxt;
  auto step = [&](auto pb, int it) {
    constexpr int PB = decltype(pb)::value;
    const uint64_t mw = mw_nxt;
    __builtin_amdgcn_s_waitcnt(0);  // this wave's asynchronous tile copies of the previous iteration have landed
    __syncthreads();                // ... and everyone's; every wave is also done with the buffers refilled below
    __bf16* const k_cur = PB ? k_s1 : k_s0;
    __bf16* const k_oth = PB ? k_s0 : k_s1;
    __bf16* const v_cur = PB ? v_s1 : v_s0;
    __bf16* const v_oth = PB ? v_s0 : v_s1;
    // a partial tile in which none of this wave's 32 queries sees a key adds exact zeros: such a wave only takes part
    // in the copies and barriers of the step (not in the dense-tile baseline, which stands for a kernel that knows
    // nothing about the mask's structure)
    const bool live = (e0 >> 31) != 0 || (SCHED == 0 && P.mode == BBM_MODE_DENSE_BASELINE) || __ballot(mw != 0ull) != 0ull;
    f32x16 s[2];
    // Wave priority: the two phases that feed the matrix pipe are raised above the address arithmetic, copy requests
    // and maxima of the other waves on the SIMD, so a wave that has matrix work issues it first (dense masks: d=64
    // -3 %, d=128 -1.5 %; neutral on the short rows of packed sequences).
    __builtin_amdgcn_s_setprio(2);
    if (live) qk(k_cur, s);
    __builtin_amdgcn_s_setprio(0);
    // the next tile's copies are requested behind the first product: their address arithmetic runs while the matrix
    // pipe works (about 1 % on dense masks)
    if (e1 != kNoTile) {
      load_tile_async(Kg, tile_of(e1), k_oth, KBLK);
      load_tile_async(Vg, tile_of(e1), v_oth, VBLK);
      if ((e1 >> 30) == 0) mw_nxt = mrow[(int64_t)tile_of(e1) * N];
      else mw_nxt = 0;
    }

    if (live) {
      // ---- element mask (only where the schedule cannot rule out zeros): keep s where the bit is set, else -inf
      if ((e0 >> 31) == 0) {
  #pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const uint32_t w = (uint32_t)(mw >> (32 * kb)) >> (4 * hh);
  #pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int bit = 8 * (e / 4) + (e % 4);
            const uint32_t keep = (uint32_t)((int32_t)(w << (31 - bit)) >> 31);  // all ones iff the bit is set
            s[kb][e] = __uint_as_float((__float_as_uint(s[kb][e]) & keep) | (0xff800000u & ~keep));
          }
        }
      }

      // ---- row maximum of this lane's query row
      float mx = s[0][0];
  #pragma unroll
      for (int kb = 0; kb < 2; ++kb)
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[kb][e]);
      mx = partner_max(mx);
      // The scores arrive relative to the reference (s = exponent - m_run).  The reference only moves when some row's
      // maximum exceeds it by more than kLazy: softmax is invariant to the reference, probabilities stay <= 2^kLazy, and
      // the rescale of O -- and here also the per-element subtraction -- is skipped on almost every tile.
      if (__any(((m_run == -INFINITY) ? (mx > -INFINITY) : (mx > kLazy)) ? 1 : 0)) {
        const float m_old = (m_run == -INFINITY) ? 0.0f : m_run;       // what the accumulators started from
        const float m_new = fmaxf(m_run, m_old + mx);
        const float m_fin = (m_new == -INFINITY) ? 0.0f : m_new;
        const float alpha = ex2(m_run - m_fin);
        const float shift = m_fin - m_old;
        l_run *= alpha;
        m_run = m_new;
  #pragma unroll
        for (int e = 0; e < 16; ++e) s_init[e] = -m_fin;
  #pragma unroll
        for (int kb = 0; kb < 2; ++kb)
          for (int e = 0; e < 16; ++e) s[kb][e] -= shift;
  #pragma unroll
        for (int db = 0; db < DB; ++db)
          for (int e = 0; e < 16; ++e) oacc[db][e] *= alpha;
      }

      __builtin_amdgcn_s_setprio(1);
  #pragma unroll
      for (int u = 0; u < 4; ++u) {
        bf16x8 pf;
  #pragma unroll
        for (int e = 0; e < 8; ++e) pf[e] = (__bf16)ex2(s[u / 2][8 * (u % 2) + e]);
        // row sum of the ROUNDED probabilities (the same numbers the second product consumes), two per instruction
  #pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const bf16x2 pair = {pf[e], pf[e + 1]};
          l_run = __builtin_amdgcn_fdot2_f32_bf16(pair, ones2, l_run, false);
        }
        // ---- O^T += V^T P^T
  #pragma unroll
        for (int db = 0; db < DB; ++db) oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_frag(v_cur, u, db), pf, oacc[db], 0, 0, 0);
      }
      __builtin_amdgcn_s_setprio(0);
    }
    e0 = e1;
    e1 = tiles_s[it + 2];
  };

  // Starts the asynchronous copies of a window's first tile e (into buffer 0) and asks for its mask word.
  auto start_tile0 = [&](uint32_t e) {
    e0 = e;
    mw_nxt = 0;
    load_tile_async(Kg, tile_of(e0), k_s0, KBLK);
    load_tile_async(Vg, tile_of(e0), v_s0, VBLK);
    if ((e0 >> 30) == 0) mw_nxt = mrow[(int64_t)tile_of(e0) * N];
  };

  // Runs the tiles listed in tiles_s[0 .. count) (followed by sentinels) through the pipeline; `started` says that
  // start_tile0 was already called for tiles_s[0].
  auto run_window = [&](int count, bool started) {
    if (!started) start_tile0(tiles_s[0]);
    if (Q_VIA_LDS && q_pending) {  // first window of a block row: Q fragments out of the staging slab
      __builtin_amdgcn_s_waitcnt(0);  // this wave's own copies have landed (no other wave touches its slab)
      const __bf16* stage = q_stage();
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        qf[t] = *reinterpret_cast<const bf16x8*>(stage + lq * D + (((2 * t + hh) ^ (lq % RC)) * 8));
        for (int e = 0; e < 8; ++e) qf[t][e] = (__bf16)((float)qf[t][e] * c);
      }
      q_pending = false;
    }
    e1 = tiles_s[1];
    for (int it = 0; it < count; it += 2) {
      step(IntC<0>{}, it);
      if (it + 1 < count) step(IntC<1>{}, it + 1);
    }
    __syncthreads();  // whoever comes next rewrites the tile list and the K/V buffers
  };

  // Runs nt >= 1 consecutive list entries, the first of which is already known: its copies start before the list
  // itself has been fetched.
  auto run_list = [&](const uint32_t* __restrict__ list, int nt, uint32_t first) {
    start_tile0(first);
    for (int w0 = 0; w0 < nt; w0 += kWin) {
      const int count = min(kWin, nt - w0);
      for (int t = tid; t < count; t += NT) tiles_s[t] = list[w0 + t];
      if (tid < 3) tiles_s[count + tid] = kNoTile;
      __syncthreads();
      run_window(count, w0 == 0);
    }
  };

  // normalise, round to bf16, store; fully masked rows give O = 0, lse = -inf.  The wave's 32 x D output slab goes
  // through LDS (the tile buffers are idle here: two slabs fit in each) so that the global stores are whole rows:
  // 16-byte chunk ch of row r sits at chunk position ch ^ (r % RC) of the row.
  auto write_output = [&]() {
    if (Q_VIA_LDS && q_pending) {  // a block row without tiles: its Q copies still target the slabs staged in below
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      q_pending = false;
    }
    const float l_tot = partner_sum(l_run);
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    __bf16* const stage = ((wave >> 1) == 0 ? k_s0 : (wave >> 1) == 1 ? k_s1 : (wave >> 1) == 2 ? v_s0 : v_s1) + (wave & 1) * 32 * D;
    // lane coordinates, re-derived behind an optimisation barrier: otherwise the per-lane staging addresses are
    // hoisted to the kernel's start and occupy registers throughout the tile loop
    int lqo = lq, hho = hh, gro = g_row, gco = g_chunk;
    asm volatile("" : "+v"(lqo), "+v"(hho), "+v"(gro), "+v"(gco));
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 ov;
        for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(oacc[db][4 * g + e] * inv);
        *reinterpret_cast<bf16x4*>(stage + lqo * D + (((4 * db + g) ^ (lqo % RC)) * 8) + 4 * hho) = ov;
      }
    }
    const int64_t row0 = (int64_t)i * BR + wave * 32;
    __bf16* og = P.o + head_off + row0 * D;
#pragma unroll
    for (int n = 0; n < 32 / RPB; ++n) {
      const int r = n * RPB + gro;
      const bf16x8 ov = *reinterpret_cast<const bf16x8*>(stage + r * D + ((gco ^ (r % RC)) * 8));
      if (row0 + r < N) *reinterpret_cast<bf16x8*>(og + r * D + gco * 8) = ov;
    }
    if (q_ok && P.lse && hh == 0)
      P.lse[(int64_t)bh * N + qrow] = l_tot > 0.0f ? m_run * (rr / kLog2e) + __logf(l_tot) : -INFINITY;
  };

  // ---- LIST mode on a small launch: work-group = (block row, part); the parts of a row run side by side and the last
  // one to finish merges them in part order (same arithmetic as the parts of a cut row)
  if constexpr (SCHED == 2) {
    const int S = P.split;
    const int part = (int)blockIdx.x % S, rest = (int)blockIdx.x / S;
    bh = rest / P.nbr;
    i = P.nbr - 1 - (rest - bh * P.nbr);
    m = (P.Mb == 1) ? 0 : bh / P.H;
    const int hb = (P.Mb == 1) ? bh : bh - m * P.H;
    begin_item();
    if (P.mode == BBM_MODE_LIST) {  // equal shares of the row's list
      const int32_t* rp = P.row_ptr + (int64_t)m * (P.nbr + 1) + i;
      const int p_row = rp[0], n_row = rp[1] - rp[0];
      const int chunk = (n_row + S - 1) / S;
      const int p0 = p_row + part * chunk, nt = max(0, min(chunk, n_row - part * chunk));
      const uint32_t* __restrict__ list = P.col_idx + (int64_t)m * P.nbr * P.nbc + p0;
      if (nt > 0) run_list(list, nt, list[0]);
    } else {  // BITMAP, RUNS: equal shares of the block columns
      const int chunk = (P.nbc + S - 1) / S;
      const int clo = part * chunk, chi = min(P.nbc, clo + chunk);
      const int nwin = num_windows(P, m, i, clo, chi);
      for (int win = 0; win < nwin; ++win) {
        const int count = build_window<NW>(P, m, i, win, tiles_s, cnt_s, clo, chi);
        if (count > 0) run_window(count, false);
      }
    }
    if (Q_VIA_LDS && q_pending) {  // nothing was computed: let the Q copies land before anyone reuses the slabs
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      q_pending = false;
    }
    const int row = m * P.nbr + i;
    float* rec = P.partials + (((int64_t)row * S + part) * P.hbp + hb) * ((REGS + 2) * NT) + tid;
#pragma unroll
    for (int db = 0; db < DB; ++db)
      for (int e = 0; e < 16; ++e) rec[(db * 16 + e) * NT] = oacc[db][e];
    rec[REGS * NT] = m_run;
    rec[(REGS + 1) * NT] = l_run;
    // one thread publishes for the work-group: the barrier orders everyone's stores before its device-wide release,
    // and its acquire before everyone's reads after the second barrier (four times fewer fences than one per wave)
    __syncthreads();
    if (tid == 0) {
      __threadfence();
      const int arrived = atomicAdd(P.queue + 8 + row * P.hbp + hb, 1);
      if (arrived == S - 1) __threadfence();  // only the merging work-group has to see the others' parts
      item_s[1] = arrived;
    }
    __syncthreads();
    if (item_s[1] == S - 1) {
      const float* r0 = P.partials + ((int64_t)row * S * P.hbp + hb) * ((REGS + 2) * NT) + tid;
      const int64_t pstride = (int64_t)P.hbp * ((REGS + 2) * NT);
      float m_all = -INFINITY;
      for (int k = 0; k < S; ++k) m_all = fmaxf(m_all, r0[k * pstride + REGS * NT]);
      const float m_fin = (m_all == -INFINITY) ? 0.0f : m_all;
#pragma unroll
      for (int db = 0; db < DB; ++db)
        for (int e = 0; e < 16; ++e) oacc[db][e] = 0.0f;
      l_run = 0.0f;
      for (int k = 0; k < S; ++k) {
        const float* rk = r0 + k * pstride;
        const float wgt = ex2(rk[REGS * NT] - m_fin);
        l_run += wgt * rk[(REGS + 1) * NT];
#pragma unroll
        for (int db = 0; db < DB; ++db)
          for (int e = 0; e < 16; ++e) oacc[db][e] += wgt * rk[(db * 16 + e) * NT];
      }
      m_run = m_all;
      write_output();
      if (tid == 0) P.queue[8 + row * P.hbp + hb] = 0;  // last user of this counter: leave it zero for the next call
    }
    return;
  }

  // ---- which block row is this work-group's own?  Work-groups are handed to the 8 XCDs round-robin; give each XCD a
  // contiguous range of logical ids so the row blocks of one head (which share K and V) meet in one XCD's L2.
  // Launch order inside a group of G consecutive (batch, head) planes: rank-major, i.e. rank 0 of every plane of the
  // group, then rank 1 of every plane, ...  The hardware starts work-groups in index order as slots free up, so
  // with ranks sorted by length long rows start early everywhere and the short ones fill the tail.
  int own_bh, own_m, own_rank;
  {
    const int wg = (int)blockIdx.x;
    const int T = P.total_wgs;
    const int xcd = wg & 7, slot = wg >> 3;
    const int per = T >> 3, rem = T & 7;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + slot;
    const int grp = logical / (P.G * P.nbr), within = logical - grp * (P.G * P.nbr);
    const int g_planes = min(P.G, T / P.nbr - grp * P.G);
    own_rank = within / g_planes;
    own_bh = grp * P.G + (within - own_rank * g_planes);
    own_m = (P.Mb == 1) ? 0 : own_bh / P.H;
  }
  // LIST mode: the schedule's header (parts, split threshold) and this work-group's row record -- which block row has
  // its rank, where its list lies and how it starts -- are requested together: one round trip, not three
  int4 own_rec = make_int4(0, 0, 0, -1);
  int nparts_all = 0, split_T = 0;
  if (SCHED == 1) {
    static_assert(bbm::kSchedNParts == 0 && bbm::kSchedSplitT == 1, "the header is read as one 8-byte pair");
    const int2 hdr = *reinterpret_cast<const int2*>(P.sched);
    own_rec = *reinterpret_cast<const int4*>(P.sched + bbm::sched_order_base(P.Mb, P.nbr) +
                                             bbm::kSchedRowInts * (int64_t)(own_m * P.nbr + own_rank));
    nparts_all = hdr.x;
    split_T = hdr.y;
    // a workspace too small for the partial results of every (part, head) item: no row is computed in parts
    // (the same decision in every work-group: it depends on the header and the launch only)
    if ((int64_t)nparts_all * P.hbp > (int64_t)P.part_cap) {
      nparts_all = 0;
      split_T = 0x7fffffff;
    }
  }
  // ---- LIST mode, the first n_extra work-groups: before their own block row they serve the queue of cut-row parts
  // (nothing to do, and no cost, when the schedule cut no row)
  if (SCHED == 1 && (int)blockIdx.x < P.n_extra) {
    const int32_t* __restrict__ S = P.sched;
  const int n_items = nparts_all * P.hbp;
  // The first item of a work-group is its own index; later ones come from the queue counter, which therefore stands
  // for "n_extra items already handed out".
  int item = blockIdx.x;
  while (item < n_items) {
    int next_item = 0;
    if (tid == 0) next_item = P.n_extra + atomicAdd(P.queue, 1);  // asked now, needed after this item
    const int hb = item / nparts_all;
    const int32_t* seg = S + bbm::kSchedPartBase + (int64_t)bbm::kSchedPartInts * (item - hb * nparts_all);
    const int row = seg[0], p0 = seg[1], nt = seg[2], part = seg[3], nparts = seg[4], q_first = seg[5], rho = seg[6];
    m = row / P.nbr;
    i = row - m * P.nbr;
    bh = (P.Mb == 1) ? hb : m * P.H + hb;
    begin_item();
    run_list(P.col_idx + (int64_t)m * P.nbr * P.nbc + p0, nt, (uint32_t)seg[7]);

    {
      // ---- park the unnormalised partial result; the last part of the row to arrive merges them all
      float* rec = P.partials + ((int64_t)(q_first + part) * P.hbp + hb) * ((REGS + 2) * NT) + tid;
#pragma unroll
      for (int db = 0; db < DB; ++db)
        for (int e = 0; e < 16; ++e) rec[(db * 16 + e) * NT] = oacc[db][e];
      rec[REGS * NT] = m_run;
      rec[(REGS + 1) * NT] = l_run;
      // one thread publishes for the work-group: the barrier orders everyone's stores before its device-wide release,
      // and its acquire before everyone's reads after the second barrier (four times fewer fences than one per wave)
      __syncthreads();
      if (tid == 0) {
        __threadfence();
        const int arrived = atomicAdd(P.queue + 8 + rho * P.hbp + hb, 1);
        if (arrived == nparts - 1) __threadfence();  // only the merging work-group has to see the others' parts
        item_s[1] = arrived;
      }
      __syncthreads();
      const bool last = item_s[1] == nparts - 1;
      if (last) {
        const float* r0 = P.partials + ((int64_t)q_first * P.hbp + hb) * ((REGS + 2) * NT) + tid;
        const int64_t pstride = (int64_t)P.hbp * ((REGS + 2) * NT);
        float m_all = -INFINITY;
        for (int k = 0; k < nparts; ++k) m_all = fmaxf(m_all, r0[k * pstride + REGS * NT]);
        const float m_fin = (m_all == -INFINITY) ? 0.0f : m_all;
#pragma unroll
        for (int db = 0; db < DB; ++db)
          for (int e = 0; e < 16; ++e) oacc[db][e] = 0.0f;
        l_run = 0.0f;
        for (int k = 0; k < nparts; ++k) {  // fixed order: the result does not depend on which part came last
          const float* rk = r0 + k * pstride;
          const float wgt = ex2(rk[REGS * NT] - m_fin);
          l_run += wgt * rk[(REGS + 1) * NT];
#pragma unroll
          for (int db = 0; db < DB; ++db)
            for (int e = 0; e < 16; ++e) oacc[db][e] += wgt * rk[(db * 16 + e) * NT];
        }
        m_run = m_all;
        write_output();
        if (tid == 0) P.queue[8 + rho * P.hbp + hb] = 0;  // last user of this counter: leave it zero for the next call
      }
    }

    if (tid == 0) item_s[0] = next_item;
    __syncthreads();
    item = item_s[0];
    __syncthreads();  // everyone has read the item before thread 0 may publish another one
  }
  // the last leading work-group to leave the queue puts the two queue counters back to zero for the next call
  if (n_items > 0 && tid == 0 && atomicAdd(P.queue + 1, 1) == P.n_extra - 1) {
    P.queue[0] = 0;
    P.queue[1] = 0;
  }
  }

  {
    bh = own_bh;
    m = own_m;
    if (SCHED == 1) {
      i = own_rec.x;
      const int n_list = own_rec.z;
      begin_item();
      if (n_list <= split_T) {  // a row the schedule cut belongs to the queue
        if (n_list > 0) run_list(P.col_idx + (int64_t)m * P.nbr * P.nbc + own_rec.y, n_list, (uint32_t)own_rec.w);
        write_output();
      }
    } else {
      i = P.nbr - 1 - own_rank;  // from the last row up: long rows first for causal-like masks
      begin_item();
      const int nwin = num_windows(P, m, i, 0, P.nbc);
      for (int win = 0; win < nwin; ++win) {
        const int count = build_window<NW>(P, m, i, win, tiles_s, cnt_s, 0, P.nbc);
        if (count > 0) run_window(count, false);
      }
      write_output();
    }
  }
}


// Leading work-groups that serve the queue of cut-row parts before their own block row (LIST mode).
constexpr int kExtraWGs = 256;

constexpr size_t kQueueAlign = 256;
inline size_t queue_bytes(int64_t Mb, int64_t nbr, int64_t hbp) {
  const size_t n = (size_t)(8 + Mb * nbr * hbp) * sizeof(int32_t);
  return (n + kQueueAlign - 1) / kQueueAlign * kQueueAlign;
}
// one parked partial result: the fp32 accumulators of a work-group plus its running maximum and sum
inline size_t record_bytes(int d, int Br) { return (size_t)((d / 32 * 16 + 2) * (Br * 2)) * sizeof(float); }
// Partial results of cut rows: at most Mb*nbr cut parts exist (T >= 2 * mean list length), one record per (cut part,
// head-batch); in practice a handful of rows is cut (8 parts x 16 heads = 4.4 MB on the long-context workload), so
// the workspace asked for stops at kPartialCapBytes and a schedule that would need more is not followed (the rows
// are then computed whole: slower, same results up to the rounding order of the merge).
constexpr size_t kPartialCapBytes = 32u << 20;
inline size_t partial_bytes(int64_t Mb, int64_t nbr, int64_t hbp, int d, int Br) {
  return std::min((size_t)(Mb * nbr * hbp) * record_bytes(d, Br), kPartialCapBytes);
}

// A launch of at most kSplitUpTo work-groups leaves CUs idle or with a single work-group (a few block rows of new
// tokens against a long key/value cache; one long sequence with few heads): every block row is then computed in
// split_parts() equal parts -- as many as give every CU two work-groups, but no more than leave a part kSplitMinTiles
// block columns (twice that from kSplitWide work-groups on: with every CU already busy, parts of 16 tiles on average lost
// 5 % on a causal mask of 4096, parts of 64 gained 24-39 % from 8192 on).  A part costs a prologue, a parked partial
// result, a device-wide fence and a share of the merge: with 20 tiles per row, 8 parts were 3.5 times slower than none;
// with 260 tiles per row and 64 rows, 4 / 8 parts take 0.114 / 0.108 ms against 0.32 ms unsplit; 128 rows of 256 tiles:
// 0.265 ms unsplit, 0.154 / 0.114 / 0.144 with 2 / 4 / 8 parts; 384 and 512 rows lose 14-40 % with 2.
constexpr int kSplitUpTo = 256, kSplitWide = 128, kSplitTarget = 512, kSplitMax = 8, kSplitMinTiles = 32;
inline int split_parts(int64_t total_wgs, int64_t nbc) {
  if (total_wgs > kSplitUpTo) return 1;
  const int64_t min_tiles = total_wgs < kSplitWide ? kSplitMinTiles : 2 * kSplitMinTiles;
  const int64_t s = std::min<int64_t>(std::min<int64_t>(kSplitMax, kSplitTarget / total_wgs), nbc / min_tiles);
  return s < 2 ? 1 : (int)s;
}

template <int D, int NW, bool EXACT>
int launch(AttnParams& P, int64_t Mb, void* workspace, size_t workspace_bytes, hipStream_t s) {
  const size_t qb = queue_bytes(Mb, P.nbr, P.hbp);
  const bool have_ws = workspace && bbm::aligned(workspace, 16) && workspace_bytes >= qb + record_bytes(D, NW * 32);
  const int64_t cap = have_ws ? (int64_t)std::min<size_t>((workspace_bytes - qb) / record_bytes(D, NW * 32), 0x7fffffff) : 0;
  if (have_ws) {
    P.queue = static_cast<int32_t*>(workspace);
    P.partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + qb);
    P.part_cap = (int32_t)cap;
    // a launch too small to fill the chip computes every block row in parts (not the dense-tile baseline, which stands
    // for the plain one-program-per-query-block kernel)
    if (P.mode != BBM_MODE_DENSE_BASELINE) P.split = split_parts(P.total_wgs, P.nbc);
    while (P.split > 1 && (int64_t)P.total_wgs * P.split > cap) --P.split;  // every (row, part, head) parks a record
  }
  if (P.split > 1) {
    attn_fwd_kernel<D, NW, 2, EXACT><<<(unsigned)(P.total_wgs * P.split), NW * 64, 0, s>>>(P);
  } else if (P.mode == BBM_MODE_LIST) {
    P.n_extra = P.total_wgs < kExtraWGs ? P.total_wgs : kExtraWGs;
    attn_fwd_kernel<D, NW, 1, EXACT><<<(unsigned)P.total_wgs, NW * 64, 0, s>>>(P);
  } else {
    attn_fwd_kernel<D, NW, 0, EXACT><<<(unsigned)P.total_wgs, NW * 64, 0, s>>>(P);
  }
  return bbm::launch_status("bbm_attn_fwd");
}

}  // namespace

extern "C" __attribute__((visibility("default"))) size_t bbm_attn_fwd_workspace_bytes(int64_t B, int64_t H, int64_t N, int d, int Br, int Bc, int mode) {
  if (B < 1 || H < 1 || N < 1 || Br < 1 || Bc < 1 || (d != 64 && d != 128)) return 0;
  if (mode != BBM_MODE_LIST && mode != BBM_MODE_AUTO && mode != BBM_MODE_BITMAP && mode != BBM_MODE_RUNS) return 0;
  // sized for the larger of the two plane counts a caller may use (Mb = 1 or Mb = B): both give Mb*hbp = B*H
  // (N counts the queries; the number of keys is not known here, so the largest split of a small launch is assumed)
  const int64_t nbr = (N + Br - 1) / Br;
  const int split = split_parts(B * H * nbr, 1 << 30);
  if (split > 1) return queue_bytes(1, nbr, B * H) + (size_t)(B * H * nbr * split) * record_bytes(d, Br);
  if (mode == BBM_MODE_BITMAP || mode == BBM_MODE_RUNS) return 0;  // these only ever use it for a small launch
  return queue_bytes(1, nbr, B * H) + partial_bytes(1, nbr, B * H, d, Br);
}

// ---- Scratch of bbm_attn_fwd_static: a file-scope device array instead of a caller's workspace, for callers that
// cannot allocate.  Every GPU the library runs on holds its own copy at its own address; host code only ever uses the
// address hipGetSymbolAddress returned for the current device, never the array's name.
constexpr size_t kStaticScratchBytes = 32u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device, kept afterwards).
int static_scratch_address(const char* fn, void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return bbm::fail(BBM_EHIP, "%s: hipGetDevice: %s", fn, hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return bbm::fail(BBM_EUNSUPPORTED, "%s: device %d is beyond the %d devices the static scratch serves", fn, dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return bbm::fail(BBM_EHIP, "%s: hipGetSymbolAddress(scratch): %s", fn, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return BBM_OK;
}

// The queue counters at the head of the scratch must be zero when the attention kernel starts.  (A fill kernel, not a
// memset: a caller may be recording the stream into a graph.)
__global__ __launch_bounds__(256) void clear_counters_kernel(int32_t* counters, int n) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < n) counters[t] = 0;
}
}  // namespace

namespace {
int attn_fwd_impl(const char* fn, const void* q, const void* k, const void* v, void* o, float* lse, int64_t B, int64_t H, int64_t N, int64_t Nk,
                  int d, float softmax_scale, int64_t Mb, const uint64_t* packed_mask, const bbm_index* idx, int mode,
                  void* workspace, size_t workspace_bytes, void* stream, bool use_static) {
  using namespace bbm;
  clear_error();
  if (!q || !k || !v || !o) return fail(BBM_EINVAL, "%s: q, k, v, o must not be NULL", fn);
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16))
    return fail(BBM_EINVAL, "%s: q, k, v, o must be 16-byte aligned", fn);
  if (lse && !aligned(lse, 4)) return fail(BBM_EINVAL, "%s: lse must be 4-byte aligned", fn);
  if (B < 1 || H < 1 || N < 1 || Nk < 1)
    return fail(BBM_EINVAL, "%s: B=%lld, H=%lld, N=%lld (queries), %lld (keys) must be >= 1", fn, (long long)B, (long long)H, (long long)N, (long long)Nk);
  if (!(softmax_scale > 0.0f) || !(softmax_scale < INFINITY)) return fail(BBM_EINVAL, "%s: softmax_scale must be finite and > 0", fn);
  if (Mb != 1 && Mb != B) return fail(BBM_EINVAL, "%s: Mb=%lld must be 1 or B=%lld", fn, (long long)Mb, (long long)B);
  if (!idx) return fail(BBM_EINVAL, "%s: idx must not be NULL", fn);
  if (!packed_mask || !aligned(packed_mask, 8)) return fail(BBM_EINVAL, "%s: packed_mask must be a non-NULL 8-byte aligned pointer", fn);
  if (d != 64 && d != 128) return fail(BBM_EUNSUPPORTED, "%s: d=%d has no kernel instance (64, 128)", fn, d);
  if (idx->Bc != kBc || (idx->Br != 64 && idx->Br != 128 && idx->Br != 256))
    return fail(BBM_EUNSUPPORTED, "%s: tile (Br=%d, Bc=%d) has no kernel instance (Br in {64,128,256}, Bc = 64)", fn, idx->Br, idx->Bc);
  const int64_t nbr = ceil_div(N, idx->Br), nbc = ceil_div(Nk, idx->Bc);
  if (idx->Nq != N || idx->Nk != Nk)
    return fail(BBM_EINVAL, "%s: index built for a mask of %lld x %lld does not match %lld queries x %lld keys", fn, (long long)idx->Nq,
                (long long)idx->Nk, (long long)N, (long long)Nk);
  if (idx->Mb != Mb || idx->nbr != nbr || idx->nbc != nbc)
    return fail(BBM_EINVAL, "%s: index (Mb=%lld, nbr=%lld, nbc=%lld) does not match the problem (Mb=%lld, nbr=%lld, nbc=%lld)", fn,
                (long long)idx->Mb, (long long)idx->nbr, (long long)idx->nbc, (long long)Mb, (long long)nbr, (long long)nbc);
  if (mode == BBM_MODE_AUTO)
    mode = (idx->row_ptr && idx->col_idx && idx->sched) ? BBM_MODE_LIST
           : (idx->bin_blk_mat && idx->offset && idx->total_ones && idx->nz_lo && idx->nz_hi) ? BBM_MODE_RUNS
                                                                                              : BBM_MODE_BITMAP;
  switch (mode) {
    case BBM_MODE_BITMAP:
      if (!idx->bin_blk_mat) return fail(BBM_EINVAL, "%s: BITMAP mode needs idx->bin_blk_mat", fn);
      break;
    case BBM_MODE_RUNS:
      if (!idx->bin_blk_mat || !idx->offset || !idx->total_ones || !idx->nz_lo || !idx->nz_hi)
        return fail(BBM_EINVAL, "%s: RUNS mode needs bin_blk_mat, offset, total_ones, nz_lo, nz_hi", fn);
      break;
    case BBM_MODE_LIST:
      if (!idx->row_ptr || !idx->col_idx || !idx->sched)
        return fail(BBM_EINVAL, "%s: LIST mode needs row_ptr, col_idx and sched", fn);
      break;
    case BBM_MODE_DENSE_BASELINE:
      // empty blocks have no packed words in memory: the kernel takes their zeros from the class bytes
      if (!idx->bin_blk_mat && !idx->blk_class) return fail(BBM_EINVAL, "%s: DENSE_BASELINE mode needs idx->bin_blk_mat or idx->blk_class", fn);
      break;
    default:
      return fail(BBM_EINVAL, "%s: unknown mode %d", fn, mode);
  }
  if (nbr * nbc >= (1ll << 31) || B * H * nbr >= (1ll << 31) || N >= (1ll << 31) || Nk >= (1ll << 31))
    return fail(BBM_EUNSUPPORTED, "%s: problem too large for 32-bit tile counters", fn);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (use_static) {
    workspace = nullptr;
    workspace_bytes = 0;
    if (mode == BBM_MODE_LIST || (mode != BBM_MODE_DENSE_BASELINE && split_parts(B * H * nbr, nbc) > 1)) {
      // the counters and at least one partial result per (batch, head) must fit; what else fits decides whether cut
      // rows and small launches are computed in parts (see launch())
      const size_t floor_bytes = queue_bytes(Mb, nbr, Mb == 1 ? B * H : H) + record_bytes(d, idx->Br);
      if (floor_bytes > kStaticScratchBytes)
        return fail(BBM_EWORKSPACE, "%s: B*H*ceil(Nq/Br) = %lld block rows need %zu bytes of counters, beyond the static scratch of %zu bytes; "
                    "use bbm_attn_fwd_rect with a workspace", fn, (long long)(B * H * nbr), floor_bytes, kStaticScratchBytes);
      if (int rc = static_scratch_address(fn, &workspace)) return rc;
      workspace_bytes = kStaticScratchBytes;
      const int n_counters = (int)(8 + B * H * nbr);
      clear_counters_kernel<<<(unsigned)((n_counters + 255) / 256), 256, 0, s>>>(static_cast<int32_t*>(workspace), n_counters);
      if (int rc = launch_status(fn)) return rc;
    }
  } else {
    // LIST mode cannot do without its workspace; BITMAP and RUNS use one, if given, to compute a small launch in parts
    const size_t need = mode == BBM_MODE_LIST ? bbm_attn_fwd_workspace_bytes(B, H, N, d, idx->Br, idx->Bc, mode) : 0;
    if (need > 0 && (!workspace || workspace_bytes < need))
      return fail(BBM_EWORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? workspace_bytes : (size_t)0);
    if (need > 0 && !aligned(workspace, 16)) return fail(BBM_EINVAL, "%s: workspace must be 16-byte aligned", fn);
  }

  AttnParams P;
  P.q = static_cast<const __bf16*>(q);
  P.k = static_cast<const __bf16*>(k);
  P.v = static_cast<const __bf16*>(v);
  P.o = static_cast<__bf16*>(o);
  P.lse = lse;
  P.packed = packed_mask;
  P.bin_blk_mat = idx->bin_blk_mat ? idx->bin_blk_mat : idx->blk_class;  // either is zero exactly on empty blocks
  P.offset = idx->offset;
  P.total_ones = idx->total_ones;
  P.nz_lo = idx->nz_lo;
  P.nz_hi = idx->nz_hi;
  P.row_ptr = idx->row_ptr;
  P.col_idx = idx->col_idx;
  P.N = N;
  P.Nk = Nk;
  P.H = (int32_t)H;
  P.Mb = (int32_t)Mb;
  P.nbr = (int32_t)nbr;
  P.nbc = (int32_t)nbc;
  P.W = (int32_t)ceil_div(Nk, 64);
  P.total_wgs = (int32_t)(B * H * nbr);
  P.mode = mode;
  // scales up to the usual 1/sqrt(d) fold into the bf16 Q; sharper ones keep the non-power-of-two part in fp32
  const float c = softmax_scale * kLog2e;
  const bool exact = softmax_scale * sqrtf((float)d) > 1.0f + 1.0f / 1024.0f;
  int c_exp = 0;
  (void)frexpf(c, &c_exp);                       // c = f * 2^c_exp, f in [0.5, 1)
  P.qscale = exact ? ldexpf(1.0f, c_exp - 1) : c;
  P.rmul = exact ? c / P.qscale : 1.0f;         // in [1, 2)
  P.sched = idx->sched;
  P.queue = nullptr;
  P.partials = nullptr;
  P.hbp = (int32_t)(Mb == 1 ? B * H : H);
  P.n_extra = 0;
  P.split = 1;
  P.part_cap = 0;
  P.G = interleaved_planes(B * H, 2 * Nk * d * (int64_t)sizeof(__bf16));
  auto go = [&](auto ex) {
    constexpr bool EX = decltype(ex)::value != 0;
    if (d == 64) {
      if (idx->Br == 64) return launch<64, 2, EX>(P, Mb, workspace, workspace_bytes, s);
      if (idx->Br == 128) return launch<64, 4, EX>(P, Mb, workspace, workspace_bytes, s);
      return launch<64, 8, EX>(P, Mb, workspace, workspace_bytes, s);
    }
    if (idx->Br == 64) return launch<128, 2, EX>(P, Mb, workspace, workspace_bytes, s);
    if (idx->Br == 128) return launch<128, 4, EX>(P, Mb, workspace, workspace_bytes, s);
    return launch<128, 8, EX>(P, Mb, workspace, workspace_bytes, s);
  };
  return exact ? go(IntC<1>{}) : go(IntC<0>{});
}
}  // namespace

extern "C" __attribute__((visibility("default"))) int bbm_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B, int64_t H,
                            int64_t N, int d, float softmax_scale, int64_t Mb, const uint64_t* packed_mask,
                            const bbm_index* idx, int mode, void* workspace, size_t workspace_bytes, void* stream) {
  return attn_fwd_impl("bbm_attn_fwd", q, k, v, o, lse, B, H, N, N, d, softmax_scale, Mb, packed_mask, idx, mode, workspace, workspace_bytes, stream, false);
}

extern "C" __attribute__((visibility("default"))) int bbm_attn_fwd_rect(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B,
                                 int64_t H, int64_t Nq, int64_t Nk, int d, float softmax_scale, int64_t Mb,
                                 const uint64_t* packed_mask, const bbm_index* idx, int mode, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  return attn_fwd_impl("bbm_attn_fwd_rect", q, k, v, o, lse, B, H, Nq, Nk, d, softmax_scale, Mb, packed_mask, idx, mode, workspace, workspace_bytes,
                       stream, false);
}

extern "C" __attribute__((visibility("default"))) int bbm_attn_fwd_static(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B,
                                   int64_t H, int64_t Nq, int64_t Nk, int d, float softmax_scale, int64_t Mb,
                                   const uint64_t* packed_mask, const bbm_index* idx, int mode, void* stream) {
  return attn_fwd_impl("bbm_attn_fwd_static", q, k, v, o, lse, B, H, Nq, Nk, d, softmax_scale, Mb, packed_mask, idx, mode, nullptr, 0, stream, true);
}
