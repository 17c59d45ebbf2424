// Backward pass of the fused masked attention (paper Sec. 3 "Flash Attention": the attention matrix is recomputed in
// the backward pass; Sec. 4: only non-zero blocks are visited and the element mask is applied only on partial ones).
//
// With P = softmax over the allowed keys (recomputed from the stored log-sum-exp), dP = dO V^T, D_i = <dO_i, O_i>,
// dS = P o (dP - D):   dV = P^T dO,   dK = scale * dS^T Q,   dQ = scale * dS K.
//
// Two kernels, both deterministic (no atomics):
//   dq kernel   one work-group per block row of Br = 32*NW queries, one lane per query (the layout of the forward
//               kernel): walks the row's list of key tiles, S^T = K Q^T and dP^T = V dO^T with the tile rows as the
//               A operand, dQ^T += K^T dS^T with K read through transposing LDS reads.  It also computes D_i and
//               leaves -D_i and -lse_i*log2(e) in the workspace for the second kernel.
//   dkv kernel  one work-group (2 waves) per block column of 64 keys, one lane per key: walks the column's list of
//               query blocks in sub-tiles of 64 queries, S = Q K^T and dP = dO V^T with the tile rows as A operand,
//               dV^T += dO^T P and dK^T += Q^T dS with transposing LDS reads of the same two tiles.
// Both start the score accumulators at -lse (in exponent units) and the dP accumulators at -D, so that exp2 and one
// multiplication per element give P and dS.
#include "bbm_internal.h"

#include <algorithm>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kWin = 128;                   // list entries per LDS window
constexpr uint32_t kNoTile = 0xffffffffu;

struct BwdParams {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  const __bf16* o;
  const __bf16* d_o;
  const float* lse;
  __bf16* dq;
  __bf16* dk;
  __bf16* dv;
  float* nl2;      // workspace [B*H*N]: -lse*log2(e), -inf for fully masked rows
  float* ndelta;   // workspace [B*H*N]: -<dO_i, O_i>
  const uint64_t* packed;  // [Mb][W][N]
  const int32_t* row_ptr;
  const uint32_t* col_idx;
  const int32_t* sched;    // may be NULL: block rows are then started from the last to the first
  const int32_t* col_ptr;
  const uint32_t* row_idx;
  int64_t N;
  int32_t H, Mb, nbr, nbc, W;
  int32_t total_wgs;
  int32_t G, Gc;    // (batch, head) planes whose block rows / block columns are interleaved in launch order
  int32_t br;       // query rows per block row
  float scale;
  float qscale;  // factor folded into the bf16 Q (dQ step) resp. K (dK/dV step) operand, see the forward kernel
  float rmul;    // EXACT instances: the rest of softmax_scale*log2(e), applied in fp32 inside the exponential; else 1
  // Cut block rows (dQ) and cut block columns (dK, dV): the split schedules (read-only), and in the caller's workspace
  // the work-queue state and the fp32 partial results of the parts.  Counters: [0] part items handed out, [1] leading
  // work-groups done, [8 + rho*hbp + hb] finished parts of cut row/column rho; all zero between calls.
  const int32_t* csched;   // column schedule; may be NULL (no column is cut then)
  int32_t* row_queue;
  int32_t* col_queue;
  float* row_partials;     // [(cut part)*hbp + hb][Br*D]
  float* col_partials;     // [(cut part)*hbp + hb][2][64*D]
  int32_t hbp;             // (batch, head) pairs per mask plane
  int32_t n_extra;         // leading work-groups that serve the queue of parts before their own row/column
};

__device__ __forceinline__ float partner_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// LDS layout of a 64-row x D tile, shared by every tile of both kernels.  One asynchronous copy instruction of a wave
// fills one 1 KiB block with RPB rows that lie NBLK rows apart: row r sits in block r % NBLK at slot r / NBLK; blocks
// are 1 KiB + 64 B apart, and the 16-byte chunk c of row r sits at chunk position c ^ ((r >> 2) & 3).  With that both
// access patterns are free of bank conflicts: 16 lanes reading the same chunk of 16 consecutive rows (A operand from
// tile rows), and 32 lanes reading 64 contiguous bytes of 4 consecutive rows (transposing read).
template <int D>
struct TL {
  static constexpr int RC = D / 8;          // 16-byte chunks per row
  static constexpr int RPB = 64 / RC;       // rows per 1 KiB block
  static constexpr int NBLK = 64 / RPB;     // blocks per tile
  static constexpr int TBLK = 512 + 32;     // block stride in elements
  static constexpr int ELEMS = NBLK * TBLK;
};

// Asynchronous global -> LDS copy of rows row0 .. row0+63 of a [N][D] matrix.  Lane l of a copy instruction lands at
// block base + 16*l, i.e. slot l / RC, chunk position l % RC.  Rows past N re-read row N-1 (callers make sure such
// rows contribute nothing).
template <int D, int NW>
__device__ __forceinline__ void tile_copy_async(const __bf16* __restrict__ src, int64_t row0, int64_t N, __bf16* dst, int wave, int lane) {
  using L = TL<D>;
  constexpr int LPW = L::NBLK / NW;
  static_assert(L::NBLK % NW == 0, "tile must split evenly over the waves");
  const int slot = lane / L::RC, pos = lane % L::RC;
  const int64_t first = min(row0, N - 1);  // a tile that starts past N re-reads row N-1 throughout
  const char* tile = reinterpret_cast<const char*>(src + first * D);
  const int last = (int)min<int64_t>(63, N - 1 - first);
#pragma unroll
  for (int n = 0; n < LPW; ++n) {
    const int blk = n * NW + wave;
    const int row = blk + L::NBLK * slot;
    const int c = pos ^ ((row >> 2) & 3);
    const uint32_t off = (uint32_t)(min(row, last) * D + c * 8) * 2u;
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(tile + off),
                                     (void __attribute__((address_space(3)))*)(dst + blk * L::TBLK), 16, 0, 0);
  }
}

// Per-lane base addresses (in elements) of the two read patterns.
template <int D>
struct TileAddr {
  int ra[2];  // A operand from tile rows: row 32*blk + lane%32, chunk 2t + lane/32; ra[t & 1] + (t >> 1)*32 + blk*(32/NBLK)*D
  int ta[2];  // transposing read of 16-row step u, half a, column block db: ta[a] + u*(D == 64 ? 2*D : D) + db*32
  __device__ __forceinline__ void init(int lane) {
    using L = TL<D>;
    const int lq = lane & 31, hh = lane >> 5;
    const int hq = (lq >> 2) & 3;
    const int rowbase = (lq % L::NBLK) * L::TBLK + (lq / L::NBLK) * D;
    const int x = hh ^ (hq & 1), y = hq >> 1;
    ra[0] = rowbase + (2 * y + x) * 8;
    ra[1] = rowbase + (2 * (1 ^ y) + x) * 8;
    const int vy = (lane & 15) >> 2, vg = (lane >> 4) & 1, vx = (lane & 3) >> 1;
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      const int blockrow = D == 64 ? (4 * hh + vy) * L::TBLK + a * D : (8 * a + 4 * hh + vy) * L::TBLK;
      ta[a] = blockrow + (2 * (vg ^ a) + (vx ^ hh)) * 8 + 4 * (lane & 1);
    }
  }
  __device__ __forceinline__ bf16x8 row_frag(const __bf16* tile, int blk, int t) const {
    using L = TL<D>;
    return *reinterpret_cast<const bf16x8*>(tile + ra[t & 1] + (t >> 1) * 32 + blk * (32 / L::NBLK) * D);
  }
  // rows 16u + 8a + 4*(lane/32) + 0..3 (a = 0, 1) of column 32*db + lane%32: the order in which a lane's accumulator
  // registers 8*(u%2) .. 8*(u%2)+7 of row block u/2 list the rows of a 32x32 product
  __device__ __forceinline__ bf16x8 tr_frag(const __bf16* tile, int u, int db) const {
    s16x4 part[2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
      part[a] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (s16x4 __attribute__((address_space(3)))*)(tile + ta[a] + u * (D == 64 ? 2 * D : D) + db * 32));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7));
  }
};

// acc * mult, rounded to bf16, to rows row0 .. of a [N][D] matrix: lane l holds row l%32 of the wave's 32-row slab,
// columns 32*db + 8*(e/4) + 4*(l/32) + e%4.  The slab is staged in LDS (`stage`, 32*D elements, this wave's own) so
// that the global stores are whole rows: 16-byte chunk ch of row r sits at chunk position ch ^ (r % RC).
template <int D>
__device__ __forceinline__ void store_slab(const f32x16 (&acc)[D / 32], float mult, __bf16* stage, __bf16* __restrict__ dst,
                                           int64_t row0, int64_t N, int lane) {
  using L = TL<D>;
  const int lq = lane & 31, hh = lane >> 5, gro = lane / L::RC, gco = lane % L::RC;
#pragma unroll
  for (int db = 0; db < D / 32; ++db) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 ov;
      for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(acc[db][4 * g + e] * mult);
      *reinterpret_cast<bf16x4*>(stage + lq * D + (((4 * db + g) ^ (lq % L::RC)) * 8) + 4 * hh) = ov;
    }
  }
  __bf16* og = dst + row0 * D;
#pragma unroll
  for (int n = 0; n < 32 / L::RPB; ++n) {
    const int r = n * L::RPB + gro;
    const bf16x8 ov = *reinterpret_cast<const bf16x8*>(stage + r * D + ((gco ^ (r % L::RC)) * 8));
    if (row0 + r < N) *reinterpret_cast<bf16x8*>(og + r * D + gco * 8) = ov;
  }
}

template <int V>
struct IntC {
  static constexpr int value = V;
};

// XCD-aware logical work-group id: work-groups are handed to the 8 XCDs round-robin; give each XCD a contiguous range
// of logical ids so that the work-groups of one head (which share its tensors) meet in one XCD's L2.
__device__ __forceinline__ int logical_wg(int wg, int total) {
  const int xcd = wg & 7, slot = wg >> 3;
  const int per = total >> 3, rem = total & 7;
  return xcd * per + (xcd < rem ? xcd : rem) + slot;
}

// ------------------------------------------------------------------------------------------------------------------
// dQ (and D, and the negated statistics for the dK/dV kernel)
// ------------------------------------------------------------------------------------------------------------------
// One work-group per (block row, batch, head).  The first P.n_extra work-groups, before turning to their own block
// row, take the parts of the block rows which the split schedule cut from a queue; the work-group that completes a
// row's last part adds the parts up in part order and writes the row, and the row's own work-group only writes the
// statistics.
// EXACT (softmax scales sharper than 1/sqrt(d)): only the power-of-two part of softmax_scale*log2(e) is folded into
// the bf16 operand, the rest multiplies the recomputed score inside the exponential, as in the forward kernel.
template <int D, int NW, bool EXACT>
__global__ __launch_bounds__(NW * 64, (D == 128 && NW >= 4) ? 2 : (D == 64 && NW == 4) ? 3 : 1) void attn_bwd_dq_kernel(const BwdParams P) {
  using L = TL<D>;
  constexpr int NT = NW * 64;
  constexpr int BR = NW * 32;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int REGS = DB * 16;
  static_assert(2 * 32 * D <= L::ELEMS && NW <= 8, "two 32 x D output slabs must fit in each tile buffer");

  __shared__ __attribute__((aligned(16))) __bf16 k_s0[L::ELEMS];
  __shared__ __attribute__((aligned(16))) __bf16 k_s1[L::ELEMS];
  __shared__ __attribute__((aligned(16))) __bf16 v_s0[L::ELEMS];
  __shared__ __attribute__((aligned(16))) __bf16 v_s1[L::ELEMS];
  __shared__ uint32_t tiles_s[kWin + 4];
  __shared__ int item_s[2];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, hh = lane >> 5;
  const int64_t N = P.N;
  const float c = P.qscale;
  const float rr = EXACT ? P.rmul : 1.0f;
  auto ex2 = [&](float x) { return __builtin_amdgcn_exp2f(EXACT ? rr * x : x); };

  // ---- per-item state
  int bh, m, i;
  int64_t head_off;
  const __bf16* __restrict__ Kg;
  const __bf16* __restrict__ Vg;
  const uint64_t* __restrict__ mrow;
  bf16x8 qf[KS], dof[KS];
  f32x16 s_init, dp_init, dq[DB];
  float nl_lane = 0.0f, nd_lane = 0.0f;

  // this lane's query: Q * scale * log2(e) and dO as B operands, D = <dO, O>, the negated statistics
  auto begin_item = [&](bool write_stats) {
    head_off = (int64_t)bh * N * D;
    Kg = P.k + head_off;
    Vg = P.v + head_off;
    const int64_t qrow = (int64_t)i * BR + wave * 32 + lq;
    const bool q_ok = qrow < N;
    mrow = P.packed + (int64_t)m * P.W * N + (q_ok ? qrow : 0);
    float dsum = 0.0f;
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      bf16x8 of;
      if (q_ok) {
        const int64_t at = head_off + qrow * D + 16 * t + 8 * hh;
        qf[t] = *reinterpret_cast<const bf16x8*>(P.q + at);
        dof[t] = *reinterpret_cast<const bf16x8*>(P.d_o + at);
        of = *reinterpret_cast<const bf16x8*>(P.o + at);
      } else {
        for (int e = 0; e < 8; ++e) qf[t][e] = dof[t][e] = of[e] = (__bf16)0.0f;
      }
      for (int e = 0; e < 8; ++e) {
        dsum += (float)dof[t][e] * (float)of[e];
        qf[t][e] = (__bf16)((float)qf[t][e] * c);
      }
    }
    const float delta = partner_sum(dsum);
    const float lse_i = q_ok ? P.lse[(int64_t)bh * N + qrow] : -INFINITY;
    const float nl = (lse_i == -INFINITY) ? -INFINITY : -lse_i * (kLog2e / rr);
    if (write_stats && q_ok && hh == 0) {
      P.nl2[(int64_t)bh * N + qrow] = nl;
      P.ndelta[(int64_t)bh * N + qrow] = -delta;
    }
    nl_lane = nl;
    nd_lane = -delta;
    if constexpr (D == 64) {
      for (int e = 0; e < 16; ++e) {
        s_init[e] = nl;
        dp_init[e] = -delta;
      }
    }
#pragma unroll
    for (int db = 0; db < DB; ++db)
      for (int e = 0; e < 16; ++e) dq[db][e] = 0.0f;
  };

  TileAddr<D> A;
  A.init(lane);

  auto tile_of = [](uint32_t e) { return (int)(e & 0x7fffffffu); };
  uint32_t e0, e1;
  uint64_t mw_nxt = 0;
  auto request = [&](uint32_t e, __bf16* kd, __bf16* vd) {
    tile_copy_async<D, NW>(Kg, (int64_t)tile_of(e) * 64, N, kd, wave, lane);
    tile_copy_async<D, NW>(Vg, (int64_t)tile_of(e) * 64, N, vd, wave, lane);
    if ((e >> 31) == 0) mw_nxt = mrow[(int64_t)tile_of(e) * N];
  };

  auto step = [&](auto pb, int it) {
    constexpr int PB = decltype(pb)::value;
    const uint64_t mw = mw_nxt;
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    __bf16* const k_cur = PB ? k_s1 : k_s0;
    __bf16* const k_oth = PB ? k_s0 : k_s1;
    __bf16* const v_cur = PB ? v_s1 : v_s0;
    __bf16* const v_oth = PB ? v_s0 : v_s1;
    if (e1 != kNoTile) request(e1, k_oth, v_oth);
    // a partial tile in which none of this wave's 32 queries sees a key contributes exact zeros: skip it
    if ((e0 >> 31) != 0 || __ballot(mw != 0ull) != 0ull) {
      // the two 32-key halves of the tile one after the other (at D = 128 their accumulators do not fit side by side)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        f32x16 s, dp;
        if constexpr (D == 64) {
          s = s_init;
          dp = dp_init;
        } else {  // D = 128: registers are short, the start values are kept as two scalars per lane
          for (int e = 0; e < 16; ++e) {
            s[e] = nl_lane;
            dp[e] = nd_lane;
          }
        }
#pragma unroll
        for (int t = 0; t < KS; ++t) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.row_frag(k_cur, kb, t), qf[t], s, 0, 0, 0);
#pragma unroll
        for (int t = 0; t < KS; ++t) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.row_frag(v_cur, kb, t), dof[t], dp, 0, 0, 0);
        // element mask where the list cannot rule out zeros: masked scores become -inf, i.e. probability 0
        if ((e0 >> 31) == 0) {
          const uint32_t w = (uint32_t)(mw >> (32 * kb)) >> (4 * hh);
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int bit = 8 * (e / 4) + (e % 4);
            const uint32_t keep = (uint32_t)((int32_t)(w << (31 - bit)) >> 31);
            s[e] = __uint_as_float((__float_as_uint(s[e]) & keep) | (0xff800000u & ~keep));
          }
        }
#pragma unroll
        for (int u2 = 0; u2 < 2; ++u2) {
          bf16x8 dsf;
#pragma unroll
          for (int e = 0; e < 8; ++e) dsf[e] = (__bf16)(ex2(s[8 * u2 + e]) * dp[8 * u2 + e]);
#pragma unroll
          for (int db = 0; db < DB; ++db) dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.tr_frag(k_cur, 2 * kb + u2, db), dsf, dq[db], 0, 0, 0);
        }
      }
    }
    e0 = e1;
    e1 = tiles_s[it + 2];
  };

  // the tiles list[0 .. n_list), window by window
  auto run_list = [&](const uint32_t* __restrict__ list, int n_list) {
    for (int w0 = 0; w0 < n_list; w0 += kWin) {
      const int count = min(kWin, n_list - w0);
      for (int t = tid; t < count; t += NT) tiles_s[t] = list[w0 + t];
      if (tid < 3) tiles_s[count + tid] = kNoTile;
      __syncthreads();
      e0 = tiles_s[0];
      e1 = tiles_s[1];
      request(e0, k_s0, v_s0);
      for (int it = 0; it < count; it += 2) {
        step(IntC<0>{}, it);
        if (it + 1 < count) step(IntC<1>{}, it + 1);
      }
      __syncthreads();  // the next window rewrites the tile list and the buffers; the epilogue stages into them
    }
  };

  auto write_dq = [&]() {
    __bf16* const stage = ((wave >> 1) == 0 ? k_s0 : (wave >> 1) == 1 ? k_s1 : (wave >> 1) == 2 ? v_s0 : v_s1) + (wave & 1) * 32 * D;
    store_slab<D>(dq, P.scale, stage, P.dq + head_off, (int64_t)i * BR + wave * 32, N, lane);
  };

  // ---- which block row is this work-group's own: rank-major interleave of G (batch, head) planes, as in the forward
  int own_bh, own_m, rank;
  {
    const int logical = logical_wg((int)blockIdx.x, P.total_wgs);
    const int grp = logical / (P.G * P.nbr), within = logical - grp * (P.G * P.nbr);
    const int g_planes = min(P.G, P.total_wgs / P.nbr - grp * P.G);
    rank = within / g_planes;
    own_bh = grp * P.G + (within - rank * g_planes);
    own_m = (P.Mb == 1) ? 0 : own_bh / P.H;
  }
  int own_i, list_pos, n_list, nparts_all = 0, split_T = 0x7fffffff;
  if (P.sched) {
    const int2 hdr = *reinterpret_cast<const int2*>(P.sched);
    const int4 rec = *reinterpret_cast<const int4*>(P.sched + bbm::sched_order_base(P.Mb, P.nbr) +
                                                    bbm::kSchedRowInts * (int64_t)(own_m * P.nbr + rank));
    nparts_all = hdr.x;
    split_T = hdr.y;
    own_i = rec.x;
    list_pos = rec.y;
    n_list = rec.z;
  } else {
    own_i = P.nbr - 1 - rank;
    list_pos = P.row_ptr[(int64_t)own_m * (P.nbr + 1) + own_i];
    n_list = P.row_ptr[(int64_t)own_m * (P.nbr + 1) + own_i + 1] - list_pos;
  }

  // ---- the first n_extra work-groups serve the queue of cut-row parts (nothing to do when no row was cut)
  if (nparts_all > 0 && (int)blockIdx.x < P.n_extra) {
    const int32_t* __restrict__ S = P.sched;
    const int n_items = nparts_all * P.hbp;
    int item = blockIdx.x;  // the first item is the work-group's own index; later ones come from the counter
    while (item < n_items) {
      int next_item = 0;
      if (tid == 0) next_item = P.n_extra + atomicAdd(P.row_queue, 1);
      const int hb = item / nparts_all;
      const int32_t* seg = S + bbm::kSchedPartBase + (int64_t)bbm::kSchedPartInts * (item - hb * nparts_all);
      const int row = seg[0], p0 = seg[1], nt = seg[2], part = seg[3], nparts = seg[4], q_first = seg[5], rho = seg[6];
      m = row / P.nbr;
      i = row - m * P.nbr;
      bh = (P.Mb == 1) ? hb : m * P.H + hb;
      begin_item(false);
      run_list(P.col_idx + (int64_t)m * P.nbr * P.nbc + p0, nt);
      // park the partial sums; the last part of the row to arrive adds them all up in part order
      float* rec = P.row_partials + ((int64_t)(q_first + part) * P.hbp + hb) * (REGS * NT) + tid;
#pragma unroll
      for (int db = 0; db < DB; ++db)
        for (int e = 0; e < 16; ++e) rec[(db * 16 + e) * NT] = dq[db][e];
      // one thread publishes for the work-group: the barrier orders everyone's stores before its device-wide release,
      // and its acquire before everyone's reads after the second barrier (four times fewer fences than one per wave)
      __syncthreads();
      if (tid == 0) {
        __threadfence();
        const int arrived = atomicAdd(P.row_queue + 8 + rho * P.hbp + hb, 1);
        if (arrived == nparts - 1) __threadfence();  // only the merging work-group has to see the others' parts
        item_s[1] = arrived;
      }
      __syncthreads();
      if (item_s[1] == nparts - 1) {
        const float* r0 = P.row_partials + ((int64_t)q_first * P.hbp + hb) * (REGS * NT) + tid;
        const int64_t pstride = (int64_t)P.hbp * (REGS * NT);
#pragma unroll
        for (int db = 0; db < DB; ++db)
          for (int e = 0; e < 16; ++e) dq[db][e] = 0.0f;
        for (int k = 0; k < nparts; ++k) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
            for (int e = 0; e < 16; ++e) dq[db][e] += r0[k * pstride + (db * 16 + e) * NT];
        }
        write_dq();
        if (tid == 0) P.row_queue[8 + rho * P.hbp + hb] = 0;  // last user of this counter: zero for the next call
      }
      if (tid == 0) item_s[0] = next_item;
      __syncthreads();
      item = item_s[0];
      __syncthreads();
    }
    if (tid == 0 && atomicAdd(P.row_queue + 1, 1) == P.n_extra - 1) {  // the last leading work-group to leave
      P.row_queue[0] = 0;
      P.row_queue[1] = 0;
    }
  }

  bh = own_bh;
  m = own_m;
  i = own_i;
  begin_item(true);
  if (n_list <= split_T) {  // a row the schedule cut belongs to the queue
    run_list(P.col_idx + (int64_t)m * P.nbr * P.nbc + list_pos, n_list);
    write_dq();
  }
}

// ------------------------------------------------------------------------------------------------------------------
// dK, dV
// ------------------------------------------------------------------------------------------------------------------
// One work-group per (block column, batch, head); the first P.n_extra work-groups first serve the queue of
// the parts of cut block columns, as the dQ kernel does for cut block rows.
// RS = false: two waves, one per key half (32 keys); each computes all four products for its keys.
// RS = true: four waves, (key half) x (role).  Role 0 computes S, P and dV, role 1 computes dP, dS and dK; P (rounded to
// bf16, as the dV product consumes it) crosses from role 0 to role 1 through LDS at a barrier in the middle of a step.
// Each wave then holds one operand (K or V) and one accumulator set, about half the registers: at D = 128, where the
// tile buffers let two work-groups share a CU, that puts two waves on every SIMD instead of one, and one wave's
// exponentials and LDS reads run under the other's matrix products.
template <int D, bool RS, bool EXACT>
__global__ __launch_bounds__(RS ? 256 : 128, RS ? 2 : 1) void attn_bwd_dkv_kernel(const BwdParams P) {
  using L = TL<D>;
  constexpr int NW = RS ? 4 : 2, NT = 64 * NW;
  constexpr int NTP = 128;  // lanes per role: stride of the parked records
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int REGS = DB * 16;
  static_assert(2 * 32 * D <= L::ELEMS, "two 32 x D output slabs must fit in a tile buffer");

  __shared__ __attribute__((aligned(16))) __bf16 q_s0[L::ELEMS];
  __shared__ __attribute__((aligned(16))) __bf16 q_s1[L::ELEMS];
  __shared__ __attribute__((aligned(16))) __bf16 g_s0[L::ELEMS];  // dO tiles
  __shared__ __attribute__((aligned(16))) __bf16 g_s1[L::ELEMS];
  __shared__ __attribute__((aligned(16))) float nl_s0[64];
  __shared__ __attribute__((aligned(16))) float nl_s1[64];
  __shared__ __attribute__((aligned(16))) float nd_s0[64];
  __shared__ __attribute__((aligned(16))) float nd_s1[64];
  __shared__ __attribute__((aligned(16))) uint32_t mk_s0[2][64];  // [key half][query row of the sub-tile]
  __shared__ __attribute__((aligned(16))) uint32_t mk_s1[2][64];
  __shared__ uint32_t tiles_s[kWin];
  __shared__ int item_s[2];
  __shared__ __attribute__((aligned(16))) bf16x8 p_s[RS ? 2 : 1][4][64];  // RS: P of [key half][16-query step][lane]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kh = wave & 1;              // key half of the column block
  const int role = RS ? wave >> 1 : 0;  // RS: 0 = S, P, dV; 1 = dP, dS, dK
  const int lq = lane & 31, hh = lane >> 5;
  const int64_t N = P.N;
  const float c = P.qscale;
  const float rr = EXACT ? P.rmul : 1.0f;
  auto ex2 = [&](float x) { return __builtin_amdgcn_exp2f(EXACT ? rr * x : x); };

  // ---- per-item state
  int bh, m, j;
  int64_t head_off;
  const __bf16* __restrict__ Qg;
  const __bf16* __restrict__ Gg;
  const float* __restrict__ nlg;
  const float* __restrict__ ndg;
  const uint32_t* __restrict__ mcol;
  bf16x8 kf[KS], vf[KS];  // RS: kf is the wave's one operand (role 0: K scaled, role 1: V), vf unused
  f32x16 dk[DB], dv[DB];  // RS: dk is the wave's one accumulator set (role 0: dV, role 1: dK), dv unused

  // this lane's key: K * scale * log2(e) and V as B operands (keys past N: zeros, never stored)
  auto begin_item = [&]() {
    head_off = (int64_t)bh * N * D;
    Qg = P.q + head_off;
    Gg = P.d_o + head_off;
    nlg = P.nl2 + (int64_t)bh * N;
    ndg = P.ndelta + (int64_t)bh * N;
    // this wave's 32-bit half of the packed mask words of block column j (one word per query row)
    mcol = reinterpret_cast<const uint32_t*>(P.packed + ((int64_t)m * P.W + j) * N) + kh;
    const int64_t krow = (int64_t)j * 64 + kh * 32 + lq;
    const bool k_ok = krow < N;
    if constexpr (RS) {
      const __bf16* __restrict__ src = role == 0 ? P.k : P.v;
      const float mult = role == 0 ? c : 1.0f;  // exact for V
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        if (k_ok)
          kf[t] = *reinterpret_cast<const bf16x8*>(src + head_off + krow * D + 16 * t + 8 * hh);
        else
          for (int e = 0; e < 8; ++e) kf[t][e] = (__bf16)0.0f;
        for (int e = 0; e < 8; ++e) kf[t][e] = (__bf16)((float)kf[t][e] * mult);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db)
        for (int e = 0; e < 16; ++e) dk[db][e] = 0.0f;
    } else {
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        if (k_ok) {
          const int64_t at = head_off + krow * D + 16 * t + 8 * hh;
          kf[t] = *reinterpret_cast<const bf16x8*>(P.k + at);
          vf[t] = *reinterpret_cast<const bf16x8*>(P.v + at);
        } else {
          for (int e = 0; e < 8; ++e) kf[t][e] = vf[t][e] = (__bf16)0.0f;
        }
        for (int e = 0; e < 8; ++e) kf[t][e] = (__bf16)((float)kf[t][e] * c);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db)
        for (int e = 0; e < 16; ++e) dk[db][e] = dv[db][e] = 0.0f;
    }
  };

  TileAddr<D> A;
  A.init(lane);

  const int qs_shift = P.br == 64 ? 0 : P.br == 128 ? 1 : 2;  // 64-query sub-tiles per block row: 1, 2, 4
  // Requests sub-tile `sub` of list entry e into the buffers of one parity: Q and dO tiles, the negated statistics of
  // its 64 queries (-lse*log2 e and -D: one wave each), and the two 32-bit halves of the mask words if the block is
  // partial (the waves of role 0, each its own half).  Query rows past N get -inf / 0 so that their probabilities are
  // exactly 0.
  auto request = [&](uint32_t e, int sub, __bf16* qd, __bf16* gd, float* nld, float* ndd, uint32_t (*mkd)[64]) {
    const int64_t row0 = ((int64_t)(e & 0x7fffffffu) << qs_shift) * 64 + (int64_t)sub * 64;
    tile_copy_async<D, NW>(Qg, row0, N, qd, wave, lane);
    tile_copy_async<D, NW>(Gg, row0, N, gd, wave, lane);
    const int64_t r = row0 + lane;
    const bool lse_wave = wave == 0, delta_wave = wave == (RS ? 2 : 1);  // one wave of each role when the roles are split
    if (lse_wave || delta_wave) {
      float* const sd = lse_wave ? nld : ndd;
      const float* const sg = lse_wave ? nlg : ndg;
      if (r < N)
        __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(sg + r),
                                         (void __attribute__((address_space(3)))*)sd, 4, 0, 0);
      else
        sd[lane] = lse_wave ? -INFINITY : 0.0f;
    }
    if (role == 0 && (e >> 31) == 0) {
      const int64_t rc = min(r, N - 1);
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(mcol + 2 * rc),
                                       (void __attribute__((address_space(3)))*)mkd[kh], 4, 0, 0);
    }
  };

  int n_steps = 0;
  auto entry_of = [&](int s) { return tiles_s[s >> qs_shift]; };
  auto step = [&](auto pb, int s) {
    constexpr int PB = decltype(pb)::value;
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    __bf16* const q_cur = PB ? q_s1 : q_s0;
    __bf16* const g_cur = PB ? g_s1 : g_s0;
    const float* const nl_cur = PB ? nl_s1 : nl_s0;
    const float* const nd_cur = PB ? nd_s1 : nd_s0;
    const uint32_t(*mk_cur)[64] = PB ? mk_s1 : mk_s0;
    const uint32_t e0 = entry_of(s);
    if (s + 1 < n_steps) {
      const uint32_t e1 = entry_of(s + 1);
      const int sub1 = (s + 1) & ((1 << qs_shift) - 1);
      if (PB)
        request(e1, sub1, q_s0, g_s0, nl_s0, nd_s0, mk_s0);
      else
        request(e1, sub1, q_s1, g_s1, nl_s1, nd_s1, mk_s1);
    }
    const bool partial = (e0 >> 31) == 0;
    // a partial sub-tile in which none of the 64 queries sees one of this wave's 32 keys contributes exact zeros
    if constexpr (RS) {
      const bool live = !partial || __ballot(mk_cur[kh][lane] != 0u) != 0ull;  // the same for both roles of a key half
      f32x16 acc2[2];  // role 0: S^T, then P; role 1: dP^T
      bf16x8 pf[4];
      if (live) {
        const float* const init = role == 0 ? nl_cur : nd_cur;
        const __bf16* const rows = role == 0 ? q_cur : g_cur;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float4 a = *reinterpret_cast<const float4*>(init + 32 * qb + 8 * g + 4 * hh);
            acc2[qb][4 * g + 0] = a.x, acc2[qb][4 * g + 1] = a.y, acc2[qb][4 * g + 2] = a.z, acc2[qb][4 * g + 3] = a.w;
          }
#pragma unroll
          for (int t = 0; t < KS; ++t) acc2[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.row_frag(rows, qb, t), kf[t], acc2[qb], 0, 0, 0);
        }
        if (role == 0) {
#pragma unroll
          for (int qb = 0; qb < 2; ++qb) {
            float p[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) p[e] = ex2(acc2[qb][e]);
            if (partial) {
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                const uint4 w = *reinterpret_cast<const uint4*>(&mk_cur[kh][32 * qb + 8 * g + 4 * hh]);
                const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)ww[e], lq, 1);  // all ones iff bit lq is set
                  p[4 * g + e] = __uint_as_float(__float_as_uint(p[4 * g + e]) & keep);
                }
              }
            }
#pragma unroll
            for (int u2 = 0; u2 < 2; ++u2) {
#pragma unroll
              for (int e = 0; e < 8; ++e) pf[2 * qb + u2][e] = (__bf16)p[8 * u2 + e];
              p_s[kh][2 * qb + u2][lane] = pf[2 * qb + u2];
            }
          }
        }
      }
      __syncthreads();  // P of this step is in LDS (the next step's first barrier comes after its last reader)
      if (live) {
        const __bf16* const cols = role == 0 ? g_cur : q_cur;
        if (role != 0) {  // dS = P o dP, rounded to bf16, in place of P
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const bf16x8 pu = p_s[kh][u][lane];
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[u][e] = (__bf16)((float)pu[e] * acc2[u >> 1][8 * (u & 1) + e]);
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int db = 0; db < DB; ++db) dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.tr_frag(cols, u, db), pf[u], dk[db], 0, 0, 0);
      }
      return;
    }
    if (partial && __ballot(mk_cur[kh][lane] != 0u) == 0ull) return;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 sc, dp;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 a = *reinterpret_cast<const float4*>(nl_cur + 32 * qb + 8 * g + 4 * hh);
        const float4 b = *reinterpret_cast<const float4*>(nd_cur + 32 * qb + 8 * g + 4 * hh);
        sc[4 * g + 0] = a.x, sc[4 * g + 1] = a.y, sc[4 * g + 2] = a.z, sc[4 * g + 3] = a.w;
        dp[4 * g + 0] = b.x, dp[4 * g + 1] = b.y, dp[4 * g + 2] = b.z, dp[4 * g + 3] = b.w;
      }
#pragma unroll
      for (int t = 0; t < KS; ++t) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.row_frag(q_cur, qb, t), kf[t], sc, 0, 0, 0);
#pragma unroll
      for (int t = 0; t < KS; ++t) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.row_frag(g_cur, qb, t), vf[t], dp, 0, 0, 0);
      float p[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) p[e] = ex2(sc[e]);
      if (partial) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const uint4 w = *reinterpret_cast<const uint4*>(&mk_cur[kh][32 * qb + 8 * g + 4 * hh]);
          const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)ww[e], lq, 1);  // all ones iff bit lq is set
            p[4 * g + e] = __uint_as_float(__float_as_uint(p[4 * g + e]) & keep);
          }
        }
      }
#pragma unroll
      for (int u2 = 0; u2 < 2; ++u2) {
        bf16x8 pf, dsf;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          pf[e] = (__bf16)p[8 * u2 + e];
          dsf[e] = (__bf16)(p[8 * u2 + e] * dp[8 * u2 + e]);
        }
        const int u = 2 * qb + u2;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.tr_frag(g_cur, u, db), pf, dv[db], 0, 0, 0);
          dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.tr_frag(q_cur, u, db), dsf, dk[db], 0, 0, 0);
        }
      }
    }
  };

  // the query blocks list[0 .. n_list), window by window
  auto run_list = [&](const uint32_t* __restrict__ list, int n_list) {
    for (int w0 = 0; w0 < n_list; w0 += kWin) {
      const int count = min(kWin, n_list - w0);
      for (int t = tid; t < count; t += NT) tiles_s[t] = list[w0 + t];
      __syncthreads();
      n_steps = count << qs_shift;
      request(tiles_s[0], 0, q_s0, g_s0, nl_s0, nd_s0, mk_s0);
      for (int s = 0; s < n_steps; s += 2) {
        step(IntC<0>{}, s);
        if (s + 1 < n_steps) step(IntC<1>{}, s + 1);
      }
      __syncthreads();  // the next window rewrites the list and the buffers; the epilogue stages into them
    }
  };

  auto write_dkv = [&]() {
    const int64_t row0 = (int64_t)j * 64 + kh * 32;
    if constexpr (RS) {
      if (role == 0)
        store_slab<D>(dk, 1.0f, g_s0 + kh * 32 * D, P.dv + head_off, row0, N, lane);
      else
        store_slab<D>(dk, P.scale, q_s0 + kh * 32 * D, P.dk + head_off, row0, N, lane);
    } else {
      store_slab<D>(dk, P.scale, q_s0 + kh * 32 * D, P.dk + head_off, row0, N, lane);
      store_slab<D>(dv, 1.0f, g_s0 + kh * 32 * D, P.dv + head_off, row0, N, lane);
    }
  };
  // where this thread's sums sit in a parked record: [dK registers | dV registers][NTP lanes]
  const int rec_lane = kh * 64 + lane, rec_reg0 = (RS && role == 0) ? REGS : 0;

  int nparts_all = 0, split_T = 0x7fffffff;
  if (P.csched) {
    const int2 hdr = *reinterpret_cast<const int2*>(P.csched);
    nparts_all = hdr.x;
    split_T = hdr.y;
  }
  // ---- the first n_extra work-groups serve the queue of cut-column parts (nothing to do when no column was cut)
  if (nparts_all > 0 && (int)blockIdx.x < P.n_extra) {
    const int32_t* __restrict__ S = P.csched;
    const int n_items = nparts_all * P.hbp;
    int item = blockIdx.x;
    while (item < n_items) {
      int next_item = 0;
      if (tid == 0) next_item = P.n_extra + atomicAdd(P.col_queue, 1);
      const int hb = item / nparts_all;
      const int32_t* seg = S + bbm::kSchedPartBase + (int64_t)bbm::kSchedPartInts * (item - hb * nparts_all);
      const int col = seg[0], p0 = seg[1], nt = seg[2], part = seg[3], nparts = seg[4], q_first = seg[5], rho = seg[6];
      m = col / P.nbc;
      j = col - m * P.nbc;
      bh = (P.Mb == 1) ? hb : m * P.H + hb;
      begin_item();
      run_list(P.row_idx + (int64_t)m * P.nbr * P.nbc + p0, nt);
      float* rec = P.col_partials + ((int64_t)(q_first + part) * P.hbp + hb) * (2 * REGS * NTP) + rec_lane;
#pragma unroll
      for (int db = 0; db < DB; ++db)
        for (int e = 0; e < 16; ++e) {
          rec[(rec_reg0 + db * 16 + e) * NTP] = dk[db][e];
          if constexpr (!RS) rec[(REGS + db * 16 + e) * NTP] = dv[db][e];
        }
      // one thread publishes for the work-group: the barrier orders everyone's stores before its device-wide release,
      // and its acquire before everyone's reads after the second barrier (four times fewer fences than one per wave)
      __syncthreads();
      if (tid == 0) {
        __threadfence();
        const int arrived = atomicAdd(P.col_queue + 8 + rho * P.hbp + hb, 1);
        if (arrived == nparts - 1) __threadfence();  // only the merging work-group has to see the others' parts
        item_s[1] = arrived;
      }
      __syncthreads();
      if (item_s[1] == nparts - 1) {
        const float* r0 = P.col_partials + ((int64_t)q_first * P.hbp + hb) * (2 * REGS * NTP) + rec_lane;
        const int64_t pstride = (int64_t)P.hbp * (2 * REGS * NTP);
#pragma unroll
        for (int db = 0; db < DB; ++db)
          for (int e = 0; e < 16; ++e) dk[db][e] = dv[db][e] = 0.0f;
        for (int k = 0; k < nparts; ++k) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
            for (int e = 0; e < 16; ++e) {
              dk[db][e] += r0[k * pstride + (rec_reg0 + db * 16 + e) * NTP];
              if constexpr (!RS) dv[db][e] += r0[k * pstride + (REGS + db * 16 + e) * NTP];
            }
        }
        write_dkv();
        if (tid == 0) P.col_queue[8 + rho * P.hbp + hb] = 0;
      }
      if (tid == 0) item_s[0] = next_item;
      __syncthreads();
      item = item_s[0];
      __syncthreads();
    }
    if (tid == 0 && atomicAdd(P.col_queue + 1, 1) == P.n_extra - 1) {
      P.col_queue[0] = 0;
      P.col_queue[1] = 0;
    }
  }

  {
    // which block column is this work-group's own: rank-major interleave of G (batch, head) planes as in the dQ kernel,
    // ranks by list length (longest first) from the schedule's records
    const int logical = logical_wg((int)blockIdx.x, P.total_wgs);
    int list_pos, n_list;
    if (P.csched) {
      const int grp = logical / (P.Gc * P.nbc), within = logical - grp * (P.Gc * P.nbc);
      const int g_planes = min(P.Gc, P.total_wgs / P.nbc - grp * P.Gc);
      const int rank = within / g_planes;
      bh = grp * P.Gc + (within - rank * g_planes);
      m = (P.Mb == 1) ? 0 : bh / P.H;
      const int4 rec = *reinterpret_cast<const int4*>(P.csched + bbm::kSchedPartBase + (int64_t)bbm::kSchedPartInts * P.Mb * P.nbc +
                                                      bbm::kSchedRowInts * (int64_t)(m * P.nbc + rank));
      j = rec.x;
      list_pos = rec.y;
      n_list = rec.z;
    } else {
      bh = logical / P.nbc;
      j = logical - bh * P.nbc;
      m = (P.Mb == 1) ? 0 : bh / P.H;
      list_pos = P.col_ptr[(int64_t)m * (P.nbc + 1) + j];
      n_list = P.col_ptr[(int64_t)m * (P.nbc + 1) + j + 1] - list_pos;
    }
    if (n_list <= split_T) {  // a column the schedule cut belongs to the queue
      begin_item();
      run_list(P.row_idx + (int64_t)m * P.nbr * P.nbc + list_pos, n_list);
      write_dkv();
    }
  }
}

// Leading work-groups that serve a queue of parts before their own block row / column.
constexpr int kExtraWGs = 256;

inline size_t round256(size_t n) { return (n + 255) / 256 * 256; }
inline size_t stats_bytes(int64_t B, int64_t H, int64_t N) { return round256((size_t)(B * H * N) * sizeof(float)); }
// counters of one queue: 8 + one per (cut row or column, (batch, head) of its plane); at most nb * B*H of those
inline size_t queue_bytes(int64_t B, int64_t H, int64_t nb) { return round256((size_t)(8 + B * H * nb) * sizeof(int32_t)); }
// at most Mb*nbr row parts and Mb*nbc column parts exist (the split thresholds are at least twice the mean length):
// the partial results of all parts together are one fp32 copy of dQ, and of dK plus dV, each padded to whole blocks
inline size_t row_partial_bytes(int64_t B, int64_t H, int64_t nbr, int Br, int d) { return (size_t)(B * H * nbr) * Br * d * sizeof(float); }
inline size_t col_partial_bytes(int64_t B, int64_t H, int64_t nbc, int d) { return (size_t)(B * H * nbc) * 2 * 64 * d * sizeof(float); }

template <int D, bool EXACT>
int launch_bwd(BwdParams& P, int64_t B, int64_t H, hipStream_t s) {
  P.total_wgs = (int32_t)(B * H * P.nbr);
  P.n_extra = std::min<int32_t>(P.total_wgs, kExtraWGs);
  P.G = bbm::interleaved_planes(B * H, 2 * P.N * D * (int64_t)sizeof(__bf16));
  if (P.br == 64)
    attn_bwd_dq_kernel<D, 2, EXACT><<<(unsigned)P.total_wgs, 128, 0, s>>>(P);
  else if (P.br == 128)
    attn_bwd_dq_kernel<D, 4, EXACT><<<(unsigned)P.total_wgs, 256, 0, s>>>(P);
  else
    attn_bwd_dq_kernel<D, 8, EXACT><<<(unsigned)P.total_wgs, 512, 0, s>>>(P);
  int rc = bbm::launch_status("bbm_attn_bwd (dq)");
  if (rc != BBM_OK) return rc;
  P.total_wgs = (int32_t)(B * H * P.nbc);
  P.n_extra = std::min<int32_t>(P.total_wgs, kExtraWGs);
  P.Gc = P.G;
  constexpr bool RS = D == 128;
  attn_bwd_dkv_kernel<D, RS, EXACT><<<(unsigned)P.total_wgs, RS ? 256 : 128, 0, s>>>(P);
  return bbm::launch_status("bbm_attn_bwd (dk, dv)");
}

}  // namespace

extern "C" __attribute__((visibility("default"))) size_t bbm_attn_bwd_workspace_bytes(int64_t B, int64_t H, int64_t N, int d, int Br) {
  if (B < 1 || H < 1 || N < 1 || (d != 64 && d != 128) || (Br != 64 && Br != 128 && Br != 256)) return 0;
  const int64_t nbr = (N + Br - 1) / Br, nbc = (N + 63) / 64;
  return queue_bytes(B, H, nbr) + queue_bytes(B, H, nbc) + 2 * stats_bytes(B, H, N) + round256(row_partial_bytes(B, H, nbr, Br, d)) +
         col_partial_bytes(B, H, nbc, d);
}
extern "C" __attribute__((visibility("default"))) int bbm_attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                                                                   const float* lse, void* dq, void* dk, void* dv, int64_t B, int64_t H,
                                                                   int64_t N, int d, float softmax_scale, int64_t Mb,
                                                                   const uint64_t* packed_mask, const bbm_index* idx, void* workspace,
                                                                   size_t workspace_bytes, void* stream) {
  using namespace bbm;
  clear_error();
  if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv)
    return fail(BBM_EINVAL, "bbm_attn_bwd: q, k, v, o, d_o, lse, dq, dk, dv must not be NULL");
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(d_o, 16) || !aligned(dq, 16) ||
      !aligned(dk, 16) || !aligned(dv, 16))
    return fail(BBM_EINVAL, "bbm_attn_bwd: q, k, v, o, d_o, dq, dk, dv must be 16-byte aligned");
  if (!aligned(lse, 4)) return fail(BBM_EINVAL, "bbm_attn_bwd: lse must be 4-byte aligned");
  if (B < 1 || H < 1 || N < 1) return fail(BBM_EINVAL, "bbm_attn_bwd: B=%lld, H=%lld, N=%lld must be >= 1", (long long)B, (long long)H, (long long)N);
  if (!(softmax_scale > 0.0f) || !(softmax_scale < INFINITY)) return fail(BBM_EINVAL, "bbm_attn_bwd: softmax_scale must be finite and > 0");
  if (Mb != 1 && Mb != B) return fail(BBM_EINVAL, "bbm_attn_bwd: Mb=%lld must be 1 or B=%lld", (long long)Mb, (long long)B);
  if (!idx) return fail(BBM_EINVAL, "bbm_attn_bwd: idx must not be NULL");
  if (!packed_mask || !aligned(packed_mask, 8)) return fail(BBM_EINVAL, "bbm_attn_bwd: packed_mask must be a non-NULL 8-byte aligned pointer");
  if (d != 64 && d != 128) return fail(BBM_EUNSUPPORTED, "bbm_attn_bwd: d=%d has no kernel instance (64, 128)", d);
  if (idx->Bc != 64 || (idx->Br != 64 && idx->Br != 128 && idx->Br != 256))
    return fail(BBM_EUNSUPPORTED, "bbm_attn_bwd: tile (Br=%d, Bc=%d) has no kernel instance (Br in {64,128,256}, Bc = 64)", idx->Br, idx->Bc);
  const int64_t nbr = ceil_div(N, idx->Br), nbc = ceil_div(N, idx->Bc);
  if (idx->Nq != N || idx->Nk != N)
    return fail(BBM_EINVAL, "bbm_attn_bwd: index built for a mask of %lld x %lld does not match N=%lld", (long long)idx->Nq, (long long)idx->Nk,
                (long long)N);
  if (idx->Mb != Mb || idx->nbr != nbr || idx->nbc != nbc)
    return fail(BBM_EINVAL, "bbm_attn_bwd: index (Mb=%lld, nbr=%lld, nbc=%lld) does not match the problem (Mb=%lld, nbr=%lld, nbc=%lld)",
                (long long)idx->Mb, (long long)idx->nbr, (long long)idx->nbc, (long long)Mb, (long long)nbr, (long long)nbc);
  if (!idx->row_ptr || !idx->col_idx || !idx->col_ptr || !idx->row_idx)
    return fail(BBM_EINVAL, "bbm_attn_bwd: the index needs row_ptr, col_idx (block list) and col_ptr, row_idx (column list)");
  if (nbr * nbc >= (1ll << 31) || B * H * nbr >= (1ll << 31) || B * H * nbc >= (1ll << 31) || N >= (1ll << 31))
    return fail(BBM_EUNSUPPORTED, "bbm_attn_bwd: problem too large for 32-bit tile counters");
  const size_t need = bbm_attn_bwd_workspace_bytes(B, H, N, d, idx->Br);
  if (!workspace || workspace_bytes < need)
    return fail(BBM_EWORKSPACE, "bbm_attn_bwd: workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
  if (!aligned(workspace, 16)) return fail(BBM_EINVAL, "bbm_attn_bwd: workspace must be 16-byte aligned");

  BwdParams P;
  P.q = static_cast<const __bf16*>(q);
  P.k = static_cast<const __bf16*>(k);
  P.v = static_cast<const __bf16*>(v);
  P.o = static_cast<const __bf16*>(o);
  P.d_o = static_cast<const __bf16*>(d_o);
  P.lse = lse;
  P.dq = static_cast<__bf16*>(dq);
  P.dk = static_cast<__bf16*>(dk);
  P.dv = static_cast<__bf16*>(dv);
  // workspace: the two counter arrays first (they are what must be zero between calls), then statistics and partials
  char* ws = static_cast<char*>(workspace);
  P.row_queue = reinterpret_cast<int32_t*>(ws);
  ws += queue_bytes(B, H, nbr);
  P.col_queue = reinterpret_cast<int32_t*>(ws);
  ws += queue_bytes(B, H, nbc);
  P.nl2 = reinterpret_cast<float*>(ws);
  ws += stats_bytes(B, H, N);
  P.ndelta = reinterpret_cast<float*>(ws);
  ws += stats_bytes(B, H, N);
  P.row_partials = reinterpret_cast<float*>(ws);
  ws += round256(row_partial_bytes(B, H, nbr, idx->Br, d));
  P.col_partials = reinterpret_cast<float*>(ws);
  P.csched = idx->col_sched;
  P.hbp = (int32_t)(Mb == 1 ? B * H : H);
  P.n_extra = 0;
  P.packed = packed_mask;
  P.row_ptr = idx->row_ptr;
  P.col_idx = idx->col_idx;
  P.sched = idx->sched;
  P.col_ptr = idx->col_ptr;
  P.row_idx = idx->row_idx;
  P.N = N;
  P.H = (int32_t)H;
  P.Mb = (int32_t)Mb;
  P.nbr = (int32_t)nbr;
  P.nbc = (int32_t)nbc;
  P.W = (int32_t)ceil_div(N, 64);
  P.br = idx->Br;
  P.scale = softmax_scale;
  // the same rule as the forward (whose lse this call consumes): scales up to 1/sqrt(d) fold into the bf16 operand
  const float c = softmax_scale * kLog2e;
  const bool exact = softmax_scale * sqrtf((float)d) > 1.0f + 1.0f / 1024.0f;
  int c_exp = 0;
  (void)frexpf(c, &c_exp);
  P.qscale = exact ? ldexpf(1.0f, c_exp - 1) : c;
  P.rmul = exact ? c / P.qscale : 1.0f;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (exact) return d == 64 ? launch_bwd<64, true>(P, B, H, s) : launch_bwd<128, true>(P, B, H, s);
  return d == 64 ? launch_bwd<64, false>(P, B, H, s) : launch_bwd<128, false>(P, B, H, s);
}
