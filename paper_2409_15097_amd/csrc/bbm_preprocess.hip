// Stage 1a: mask bytes -> block classes, BinBlkMat and packed mask bits (paper Sec. 4 "Binary Block
// Masking"; Appendix A, block-based summation).  The sum of a block is only ever compared with 0 and with
// Br*Bc, so the kernel carries an OR and an AND of the non-zero bits instead of a count.
//
// One work-group (8 wavefronts) owns one block row (Br mask rows) x 1024 mask columns.  A wavefront streams
// whole 1 KiB row segments (16 B per lane, fully coalesced); each lane turns its 16 bytes into 16 bits and
// keeps a running OR / AND over the rows it sees.  The bits go to LDS as uint16 quarters of the 64-bit
// words and leave word-column major, so the global writes of the packed mask are contiguous too.
#include "bbm_internal.h"

namespace {

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kUnroll = 8;        // rows a lane has in flight
constexpr int kColsPerWG = 1024;  // 64 lanes x 16 bytes
constexpr int kWordsPerWG = kColsPerWG / 64;
constexpr int kMaxBr = 256;
constexpr int64_t kStreamFromBytes = 128ll << 20;

// 4 mask bytes -> 4 bits (bit t = byte t non-zero).
__device__ __forceinline__ uint32_t nz_nibble(uint32_t x) {
  uint32_t y = (((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u;  // bit 7 of each byte = byte != 0
  return (((y >> 7) * 0x00204081u) >> 21) & 0xfu;                      // gather bits 0,8,16,24 -> 0..3
}

// STREAM: the 16 bytes are read with a streaming (non-temporal) load.  A mask is read once and never again; one that is
// larger than the last-level cache can hold anyway would only push Q, K and V out of it on its way through.
template <bool ALIGNED, bool STREAM>
__device__ __forceinline__ uint32_t load_bits16(const uint8_t* row, int64_t col, int64_t N) {
  if (ALIGNED && col + 16 <= N) {
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4* p = reinterpret_cast<const u32x4*>(row + col);
    const u32x4 x = STREAM ? __builtin_nontemporal_load(p) : *p;
    return nz_nibble(x.x) | (nz_nibble(x.y) << 4) | (nz_nibble(x.z) << 8) | (nz_nibble(x.w) << 12);
  }
  uint32_t bits = 0;
  for (int t = 0; t < 16; ++t)
    if (col + t < N && row[col + t] != 0) bits |= 1u << t;
  return bits;
}

template <bool ALIGNED, bool STREAM = false>
__global__ __launch_bounds__(kThreads) void block_reduce_kernel(const uint8_t* __restrict__ mask, int64_t Nr, int64_t N,
                                                                int64_t row_stride, int Br, int Bc, int64_t nbr,
                                                                int64_t nbc, uint8_t* __restrict__ blk_class,
                                                                uint8_t* __restrict__ bin_blk_mat,
                                                                uint64_t* __restrict__ packed) {
  __shared__ __attribute__((aligned(8))) uint16_t stage[kWordsPerWG * (kMaxBr + 1) * 4];  // [word][row in block (+1 pad)][quarter]
  __shared__ uint32_t acc[kWaves][64];                  // per wave, per lane: any16 | all16 << 16
  __shared__ uint32_t word_any[kWordsPerWG];            // per 64-column word: does any of the block row's rows set a bit?

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = (int64_t)blockIdx.x * kColsPerWG;
  const int64_t i = blockIdx.y, m = blockIdx.z;
  const int64_t r0 = i * Br;
  const int rows = (int)((r0 + Br <= Nr) ? Br : (Nr - r0));  // real (unpadded) rows of this block row (Nr mask rows, N columns)
  const int64_t col = c0 + 16 * lane;
  const uint8_t* base = mask + (m * Nr + r0) * row_stride;
  const int BrP = Br + 1;  // padded row count: consecutive words land in different LDS banks

  uint32_t any16 = 0, all16 = 0xffffu;
  if (col < N) {
    int r = wave;
    for (; r + (kUnroll - 1) * kWaves < rows; r += kUnroll * kWaves) {  // kUnroll independent 16-byte loads in flight per lane
      uint32_t b[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) b[u] = load_bits16<ALIGNED, STREAM>(base + (int64_t)(r + u * kWaves) * row_stride, col, N);
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        any16 |= b[u];
        all16 &= b[u];
      }
      if (packed) {
        uint16_t* s = stage + ((lane >> 2) * BrP) * 4 + (lane & 3);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) s[(r + u * kWaves) * 4] = (uint16_t)b[u];
      }
    }
    for (; r < rows; r += kWaves) {
      uint32_t b = load_bits16<ALIGNED, STREAM>(base + (int64_t)r * row_stride, col, N);
      any16 |= b;
      all16 &= b;
      if (packed) stage[((lane >> 2) * BrP + r) * 4 + (lane & 3)] = (uint16_t)b;
    }
    // a wave that saw no row of this block keeps all16 = 0xffff: it is neutral in the AND below
  } else {
    all16 = 0;  // columns past N are padding: never full
    if (packed)
      for (int r = wave; r < rows; r += kWaves) stage[((lane >> 2) * BrP + r) * 4 + (lane & 3)] = 0;
  }
  if (rows < Br) all16 = 0;  // block row reaches into the zero padding below the mask
  acc[wave][lane] = any16 | (all16 << 16);
  __syncthreads();

  if (wave == 0) {
    uint32_t any_v = 0, all_v = 0xffffu;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t a = acc[w][lane];
      any_v |= a & 0xffffu;
      all_v &= a >> 16;
    }
    {  // four lanes of 16 columns make one packed word
      uint32_t w_any = any_v | __shfl_xor(any_v, 1);
      w_any |= __shfl_xor(w_any, 2);
      if ((lane & 3) == 0) word_any[lane >> 2] = w_any;
    }
    const int g = Bc / 16;  // lanes per block column
    for (int s = 1; s < g; s <<= 1) {
      any_v |= __shfl_xor(any_v, s);
      all_v &= __shfl_xor(all_v, s);
    }
    const int64_t j = col / Bc;
    if ((lane % g) == 0 && j < nbc) {
      const uint8_t cls = any_v == 0 ? BBM_BLOCK_EMPTY : (all_v == 0xffffu ? BBM_BLOCK_FULL : BBM_BLOCK_PARTIAL);
      const int64_t o = (m * nbr + i) * nbc + j;
      blk_class[o] = cls;
      if (bin_blk_mat) bin_blk_mat[o] = cls != BBM_BLOCK_EMPTY;
    }
  }

  if (packed) {
    // Words of a (block row x 64 columns) slab without a single set bit are not written: no schedule reads them (the
    // mask-everywhere baseline takes the zero from the class byte), and on sparse masks they are most of the output.
    __syncthreads();
    const int64_t W = (N + 63) / 64;
    const int64_t w0 = c0 / 64;
    const uint64_t* stage64 = reinterpret_cast<const uint64_t*>(stage);
    for (int t = threadIdx.x; t < kWordsPerWG * rows; t += kThreads) {
      const int wl = t / rows, rl = t - wl * rows;
      if (w0 + wl < W && word_any[wl] != 0) packed[(m * W + w0 + wl) * Nr + r0 + rl] = stage64[wl * BrP + rl];
    }
  }
}

}  // namespace

namespace {
int build_block_mask_impl(const char* fn, const uint8_t* mask, int64_t Mb, int64_t Nq, int64_t Nk, int64_t row_stride_bytes, int Br, int Bc,
                          uint8_t* blk_class, uint8_t* bin_blk_mat, uint64_t* packed_mask, void* stream) {
  using namespace bbm;
  clear_error();
  if (!mask || !blk_class) return fail(BBM_EINVAL, "%s: mask and blk_class must not be NULL", fn);
  if (Mb < 1 || Nq < 1 || Nk < 1)
    return fail(BBM_EINVAL, "%s: Mb=%lld, rows=%lld, columns=%lld must be >= 1", fn, (long long)Mb, (long long)Nq, (long long)Nk);
  if (row_stride_bytes < Nk) return fail(BBM_EINVAL, "%s: row_stride_bytes=%lld < columns=%lld", fn, (long long)row_stride_bytes, (long long)Nk);
  if (Br < 1 || Br > kMaxBr) return fail(BBM_EUNSUPPORTED, "%s: Br=%d outside [1, %d]", fn, Br, kMaxBr);
  if (Bc != 16 && Bc != 32 && Bc != 64 && Bc != 128 && Bc != 256) return fail(BBM_EUNSUPPORTED, "%s: Bc=%d not in {16,32,64,128,256}", fn, Bc);
  if (packed_mask && !aligned(packed_mask, 8)) return fail(BBM_EINVAL, "%s: packed_mask must be 8-byte aligned", fn);
  const int64_t nbr = ceil_div(Nq, Br), nbc = ceil_div(Nk, Bc);
  if (nbr > 65535 || Mb > 65535) return fail(BBM_EUNSUPPORTED, "%s: nbr=%lld or Mb=%lld exceeds 65535", fn, (long long)nbr, (long long)Mb);
  dim3 grid((unsigned)ceil_div(Nk, kColsPerWG), (unsigned)nbr, (unsigned)Mb);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool fast = aligned(mask, 16) && (row_stride_bytes % 16 == 0);
  // masks from kStreamFromBytes on (half the 256 MB last-level cache) are streamed: block reduction 6 % faster on a 1 GiB mask
  // and the attention kernel behind it finds more of Q, K, V still cached (whole step -2.5 % at 1 GiB, -3.5 % at 256 MiB);
  // a 64 MiB mask that is rebuilt from the cache it still sits in loses 20 % that way
  if (fast && Mb * Nq * Nk >= kStreamFromBytes)
    block_reduce_kernel<true, true><<<grid, kThreads, 0, s>>>(mask, Nq, Nk, row_stride_bytes, Br, Bc, nbr, nbc, blk_class, bin_blk_mat, packed_mask);
  else if (fast)
    block_reduce_kernel<true><<<grid, kThreads, 0, s>>>(mask, Nq, Nk, row_stride_bytes, Br, Bc, nbr, nbc, blk_class, bin_blk_mat, packed_mask);
  else
    block_reduce_kernel<false><<<grid, kThreads, 0, s>>>(mask, Nq, Nk, row_stride_bytes, Br, Bc, nbr, nbc, blk_class, bin_blk_mat, packed_mask);
  return launch_status(fn);
}
}  // namespace

extern "C" __attribute__((visibility("default"))) int bbm_build_block_mask(const uint8_t* mask, int64_t Mb, int64_t N, int64_t row_stride_bytes, int Br,
                                    int Bc, uint8_t* blk_class, uint8_t* bin_blk_mat, uint64_t* packed_mask,
                                    void* stream) {
  return build_block_mask_impl("bbm_build_block_mask", mask, Mb, N, N, row_stride_bytes, Br, Bc, blk_class, bin_blk_mat, packed_mask, stream);
}

extern "C" __attribute__((visibility("default"))) int bbm_build_block_mask_rect(const uint8_t* mask, int64_t Mb, int64_t Nq, int64_t Nk,
                                         int64_t row_stride_bytes, int Br, int Bc, uint8_t* blk_class,
                                         uint8_t* bin_blk_mat, uint64_t* packed_mask, void* stream) {
  return build_block_mask_impl("bbm_build_block_mask_rect", mask, Mb, Nq, Nk, row_stride_bytes, Br, Bc, blk_class, bin_blk_mat, packed_mask, stream);
}
