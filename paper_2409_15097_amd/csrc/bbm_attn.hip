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

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBc = 64;
constexpr int kPad = 8;  // bf16 elements of padding per LDS row (16 bytes)
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
  int64_t N;
  int32_t H, Mb, nbr, nbc, W;
  int32_t total_wgs;
  int32_t mode;
  float scale;
};

// Wave-uniform iterator over the tiles a block row visits, in ascending key order.
struct TileIter {
  int mode;
  int j, j_end;          // DENSE: next block / end.  BITMAP, RUNS: scan window [chunk base .. j_end)
  int base;              // BITMAP, RUNS: first block of the current 64-block chunk
  uint64_t nz;           // BITMAP, RUNS: unvisited non-zero blocks of the current chunk
  const uint8_t* row;    // BITMAP, RUNS: BinBlkMat row
  int run_lo, run_hi;    // RUNS: [offset, offset + total_ones)
  const uint32_t* list;  // LIST
  int p, p_end;

  __device__ __forceinline__ void load_chunk(int lane) {
    const int jj = base + lane;
    const uint8_t b = (jj >= j && jj < j_end) ? row[jj] : (uint8_t)0;
    nz = __ballot(b != 0);
  }

  __device__ __forceinline__ void init(const AttnParams& P, int m, int i, int lane) {
    mode = P.mode;
    const int64_t r = (int64_t)m * P.nbr + i;
    if (mode == BBM_MODE_DENSE_BASELINE) {
      j = 0;
      j_end = P.nbc;
    } else if (mode == BBM_MODE_LIST) {
      const int32_t* rp = P.row_ptr + (int64_t)m * (P.nbr + 1) + i;
      p = __builtin_amdgcn_readfirstlane(rp[0]);
      p_end = __builtin_amdgcn_readfirstlane(rp[1]);
      list = P.col_idx + (int64_t)m * P.nbr * P.nbc;
    } else {
      row = P.bin_blk_mat + r * P.nbc;
      j = 0;
      j_end = P.nbc;
      run_lo = run_hi = 0;
      if (mode == BBM_MODE_RUNS) {
        j = __builtin_amdgcn_readfirstlane(P.nz_lo[r]);
        j_end = __builtin_amdgcn_readfirstlane(P.nz_hi[r]);
        run_lo = __builtin_amdgcn_readfirstlane(P.offset[r]);
        run_hi = run_lo + __builtin_amdgcn_readfirstlane(P.total_ones[r]);
      }
      base = j & ~63;
      nz = 0;
      if (j < j_end) load_chunk(lane);
    }
  }

  // Returns the next visited block column (or -1) and whether the element mask must be applied there.
  __device__ __forceinline__ int next(int lane, bool& need_mask) {
    need_mask = true;
    if (mode == BBM_MODE_DENSE_BASELINE) {
      return j < j_end ? j++ : -1;
    }
    if (mode == BBM_MODE_LIST) {
      if (p >= p_end) return -1;
      const uint32_t e = __builtin_amdgcn_readfirstlane(list[p]);
      ++p;
      need_mask = (e >> 31) == 0;
      return (int)(e & 0x7fffffffu);
    }
    while (nz == 0) {
      base += 64;
      if (base >= j_end) return -1;
      load_chunk(lane);
    }
    const int jj = base + __builtin_ctzll(nz);
    nz &= nz - 1;
    if (mode == BBM_MODE_RUNS) need_mask = !(jj >= run_lo && jj < run_hi);
    return jj;
  }
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

template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void attn_fwd_kernel(const AttnParams P) {
  constexpr int NT = NW * 64;
  constexpr int BR = NW * 32;
  constexpr int LD = D + kPad;                 // LDS row stride in elements
  constexpr int CHUNKS = kBc * D / 8;          // 16-byte chunks per K (or V) tile
  constexpr int CPT = CHUNKS / NT;             // chunks per thread
  static_assert(CHUNKS % NT == 0, "tile must split evenly over the work-group");
  constexpr int KS = D / 16;                   // MFMA k-steps of the first product
  constexpr int DB = D / 32;                   // 32-wide output-column blocks of the second product

  __shared__ __attribute__((aligned(16))) __bf16 k_s[2][kBc * LD];
  __shared__ __attribute__((aligned(16))) __bf16 v_s[2][kBc * LD];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, hh = lane >> 5;

  // Work-groups are handed to the 8 XCDs round-robin; give each XCD a contiguous range of logical ids so the
  // row blocks of one head (which share K and V) meet in one XCD's L2.
  const int T = P.total_wgs;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int per = T >> 3, rem = T & 7;
  const int logical = xcd * per + (xcd < rem ? xcd : rem) + slot;
  const int bh = logical / P.nbr;
  const int i = P.nbr - 1 - (logical - bh * P.nbr);  // late (for causal-like masks: long) block rows first
  const int b = bh / P.H;
  const int m = (P.Mb == 1) ? 0 : b;

  const int64_t N = P.N;
  const int64_t head_off = (int64_t)bh * N * D;
  const __bf16* __restrict__ Kg = P.k + head_off;
  const __bf16* __restrict__ Vg = P.v + head_off;
  const int64_t qrow = (int64_t)i * BR + wave * 32 + lq;
  const bool q_ok = qrow < N;

  bf16x8 qf[KS];
#pragma unroll
  for (int t = 0; t < KS; ++t) {
    if (q_ok)
      qf[t] = *reinterpret_cast<const bf16x8*>(P.q + head_off + qrow * D + 16 * t + 8 * hh);
    else
      for (int e = 0; e < 8; ++e) qf[t][e] = (__bf16)0.0f;
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
    for (int e = 0; e < 16; ++e) oacc[db][e] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;
  const float c = P.scale * kLog2e;

  TileIter it;
  it.init(P, m, i, lane);

  uint4 kreg[CPT], vreg[CPT];
  auto load_tile = [&](int jt) {
#pragma unroll
    for (int n = 0; n < CPT; ++n) {
      const int ch = tid + n * NT;
      const int r = ch / (D / 8), cc = ch % (D / 8);
      const int64_t key = (int64_t)jt * kBc + r;
      if (key < N) {
        kreg[n] = *reinterpret_cast<const uint4*>(Kg + key * D + cc * 8);
        vreg[n] = *reinterpret_cast<const uint4*>(Vg + key * D + cc * 8);
      } else {  // keys past N: zeros, so that 0-probability times V stays 0
        kreg[n] = make_uint4(0, 0, 0, 0);
        vreg[n] = make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int n = 0; n < CPT; ++n) {
      const int ch = tid + n * NT;
      const int r = ch / (D / 8), cc = ch % (D / 8);
      *reinterpret_cast<uint4*>(&k_s[buf][r * LD + cc * 8]) = kreg[n];
      *reinterpret_cast<uint4*>(&v_s[buf][r * LD + cc * 8]) = vreg[n];
    }
  };

  bool need_mask = true, need_mask_next = true;
  int jt = it.next(lane, need_mask);
  if (jt >= 0) load_tile(jt);
  int buf = 0;
  while (jt >= 0) {
    const int jn = it.next(lane, need_mask_next);
    store_tile(buf);
    uint64_t mword = 0;
    if (need_mask && q_ok) mword = P.packed[((int64_t)m * P.W + jt) * N + qrow];
    __syncthreads();  // tile jt is in LDS; every wave is done with the other buffer's previous tile
    if (jn >= 0) load_tile(jn);

    // ---- S^T = K Q^T for 64 keys x 32 queries
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
      for (int e = 0; e < 16; ++e) s[kb][e] = 0.0f;
#pragma unroll
    for (int t = 0; t < KS; ++t) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&k_s[buf][(32 * kb + lq) * LD + 16 * t + 8 * hh]);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], s[kb], 0, 0, 0);
      }
    }

    // ---- element mask (only where the schedule cannot rule out zeros): keep s where the bit is set, else -inf
    if (need_mask) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const uint32_t w = (uint32_t)(mword >> (32 * kb)) >> (4 * hh);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int bit = 8 * (e / 4) + (e % 4);
          const uint32_t keep = (uint32_t)((int32_t)(w << (31 - bit)) >> 31);  // all ones iff the bit is set
          s[kb][e] = __uint_as_float((__float_as_uint(s[kb][e]) & keep) | (0xff800000u & ~keep));
        }
      }
    }

    // ---- online softmax for this lane's query row
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[kb][e]);
    mx = partner_max(mx);
    // The reference maximum m_run only moves when some row's maximum grew by more than kLazy (in log2 units):
    // softmax is invariant to the reference, probabilities stay <= 2^kLazy, and the rescale of O is skipped.
    if (__any((mx * c > m_run * c + kLazy) ? 1 : 0)) {
      const float m_new = fmaxf(m_run, mx);
      const float m_fin = (m_new == -INFINITY) ? 0.0f : m_new;
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_fin) * c);
      l_run *= alpha;
      m_run = m_new;
#pragma unroll
      for (int db = 0; db < DB; ++db)
        for (int e = 0; e < 16; ++e) oacc[db][e] *= alpha;
    }
    const float msc = ((m_run == -INFINITY) ? 0.0f : m_run) * c;
    float rs = 0.0f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][e], c, -msc));
        s[kb][e] = p;
        rs += p;
      }
    l_run += rs;

    // ---- O^T += V^T P^T
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      bf16x8 pf;
#pragma unroll
      for (int e = 0; e < 8; ++e) pf[e] = (__bf16)s[u / 2][8 * (u % 2) + e];
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        // transposing read: lane gets keys k0..k0+3 of column dcol; k0 = 16u + 8a + 4hh, matching the key order of pf
        const int vr = 16 * u + 4 * hh + ((lane & 15) >> 2);
        const int vc = 32 * db + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3)))*)(&v_s[buf][vr * LD + vc]));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3)))*)(&v_s[buf][(vr + 8) * LD + vc]));
        const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[db], 0, 0, 0);
      }
    }

    buf ^= 1;
    jt = jn;
    need_mask = need_mask_next;
  }

  // ---- epilogue: normalise, round to bf16, store; fully masked rows give O = 0, lse = -inf
  const float l_tot = partner_sum(l_run);
  const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
  if (q_ok) {
    __bf16* og = P.o + head_off + qrow * D;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 ov;
        for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(oacc[db][4 * g + e] * inv);
        *reinterpret_cast<bf16x4*>(og + 32 * db + 8 * g + 4 * hh) = ov;
      }
    }
    if (P.lse && hh == 0)
      P.lse[(int64_t)bh * N + qrow] = l_tot > 0.0f ? m_run * P.scale + __logf(l_tot) : -INFINITY;
  }
}

template <int D, int NW>
int launch(const AttnParams& P, hipStream_t s) {
  attn_fwd_kernel<D, NW><<<(unsigned)P.total_wgs, NW * 64, 0, s>>>(P);
  return bbm::launch_status("bbm_attn_fwd");
}

}  // namespace

extern "C" __attribute__((visibility("default"))) size_t bbm_attn_fwd_workspace_bytes(int64_t B, int64_t H, int64_t N, int d, int Br, int Bc, int mode) {
  (void)B; (void)H; (void)N; (void)d; (void)Br; (void)Bc; (void)mode;
  return 0;
}

extern "C" __attribute__((visibility("default"))) int bbm_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B, int64_t H,
                            int64_t N, int d, float softmax_scale, int64_t Mb, const uint64_t* packed_mask,
                            const bbm_index* idx, int mode, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace bbm;
  clear_error();
  (void)workspace;
  if (!q || !k || !v || !o) return fail(BBM_EINVAL, "bbm_attn_fwd: q, k, v, o must not be NULL");
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16))
    return fail(BBM_EINVAL, "bbm_attn_fwd: q, k, v, o must be 16-byte aligned");
  if (lse && !aligned(lse, 4)) return fail(BBM_EINVAL, "bbm_attn_fwd: lse must be 4-byte aligned");
  if (B < 1 || H < 1 || N < 1) return fail(BBM_EINVAL, "bbm_attn_fwd: B=%lld, H=%lld, N=%lld must be >= 1", (long long)B, (long long)H, (long long)N);
  if (!(softmax_scale > 0.0f) || !(softmax_scale < INFINITY)) return fail(BBM_EINVAL, "bbm_attn_fwd: softmax_scale must be finite and > 0");
  if (Mb != 1 && Mb != B) return fail(BBM_EINVAL, "bbm_attn_fwd: Mb=%lld must be 1 or B=%lld", (long long)Mb, (long long)B);
  if (!idx) return fail(BBM_EINVAL, "bbm_attn_fwd: idx must not be NULL");
  if (!packed_mask || !aligned(packed_mask, 8)) return fail(BBM_EINVAL, "bbm_attn_fwd: packed_mask must be a non-NULL 8-byte aligned pointer");
  if (d != 64 && d != 128) return fail(BBM_EUNSUPPORTED, "bbm_attn_fwd: d=%d has no kernel instance (64, 128)", d);
  if (idx->Bc != kBc || (idx->Br != 64 && idx->Br != 128 && idx->Br != 256))
    return fail(BBM_EUNSUPPORTED, "bbm_attn_fwd: tile (Br=%d, Bc=%d) has no kernel instance (Br in {64,128,256}, Bc = 64)", idx->Br, idx->Bc);
  const int64_t nbr = ceil_div(N, idx->Br), nbc = ceil_div(N, idx->Bc);
  if (idx->Mb != Mb || idx->nbr != nbr || idx->nbc != nbc)
    return fail(BBM_EINVAL, "bbm_attn_fwd: index (Mb=%lld, nbr=%lld, nbc=%lld) does not match the problem (Mb=%lld, nbr=%lld, nbc=%lld)",
                (long long)idx->Mb, (long long)idx->nbr, (long long)idx->nbc, (long long)Mb, (long long)nbr, (long long)nbc);
  if (mode == BBM_MODE_AUTO)
    mode = (idx->row_ptr && idx->col_idx) ? BBM_MODE_LIST
           : (idx->bin_blk_mat && idx->offset && idx->total_ones && idx->nz_lo && idx->nz_hi) ? BBM_MODE_RUNS
                                                                                              : BBM_MODE_BITMAP;
  switch (mode) {
    case BBM_MODE_BITMAP:
      if (!idx->bin_blk_mat) return fail(BBM_EINVAL, "bbm_attn_fwd: BITMAP mode needs idx->bin_blk_mat");
      break;
    case BBM_MODE_RUNS:
      if (!idx->bin_blk_mat || !idx->offset || !idx->total_ones || !idx->nz_lo || !idx->nz_hi)
        return fail(BBM_EINVAL, "bbm_attn_fwd: RUNS mode needs bin_blk_mat, offset, total_ones, nz_lo, nz_hi");
      break;
    case BBM_MODE_LIST:
      if (!idx->row_ptr || !idx->col_idx) return fail(BBM_EINVAL, "bbm_attn_fwd: LIST mode needs row_ptr and col_idx");
      break;
    case BBM_MODE_DENSE_BASELINE:
      break;
    default:
      return fail(BBM_EINVAL, "bbm_attn_fwd: unknown mode %d", mode);
  }
  if (nbr * nbc >= (1ll << 31) || B * H * nbr >= (1ll << 31) || N >= (1ll << 31))
    return fail(BBM_EUNSUPPORTED, "bbm_attn_fwd: problem too large for 32-bit tile counters");
  if (workspace_bytes < bbm_attn_fwd_workspace_bytes(B, H, N, d, idx->Br, idx->Bc, mode))
    return fail(BBM_EWORKSPACE, "bbm_attn_fwd: workspace too small");

  AttnParams P;
  P.q = static_cast<const __bf16*>(q);
  P.k = static_cast<const __bf16*>(k);
  P.v = static_cast<const __bf16*>(v);
  P.o = static_cast<__bf16*>(o);
  P.lse = lse;
  P.packed = packed_mask;
  P.bin_blk_mat = idx->bin_blk_mat;
  P.offset = idx->offset;
  P.total_ones = idx->total_ones;
  P.nz_lo = idx->nz_lo;
  P.nz_hi = idx->nz_hi;
  P.row_ptr = idx->row_ptr;
  P.col_idx = idx->col_idx;
  P.N = N;
  P.H = (int32_t)H;
  P.Mb = (int32_t)Mb;
  P.nbr = (int32_t)nbr;
  P.nbc = (int32_t)nbc;
  P.W = (int32_t)ceil_div(N, 64);
  P.total_wgs = (int32_t)(B * H * nbr);
  P.mode = mode;
  P.scale = softmax_scale;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (d == 64) {
    if (idx->Br == 64) return launch<64, 2>(P, s);
    if (idx->Br == 128) return launch<64, 4>(P, s);
    return launch<64, 8>(P, s);
  }
  if (idx->Br == 64) return launch<128, 2>(P, s);
  if (idx->Br == 128) return launch<128, 4>(P, s);
  return launch<128, 8>(P, s);
}
