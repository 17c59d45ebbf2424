// Reverse Cuthill-McKee reordering of a sparse attention mask on the GPU (paper Sec. 4 "Binary Block Masking with
// Reverse Cuthill-McKee (RCM)": the mask is treated as a graph and reordered so that fewer blocks are non-zero), and the
// gathers that apply the permutation to the mask and to Q/K/V/O rows.
//
// The ordering is the published algorithm with every choice fixed (the library header states them): neighbours of node
// i are the non-zero entries of mask row i, a component starts at its unvisited node of minimum degree (ties: smallest
// index), each breadth-first level is ordered by (position of the earliest parent, degree, index), the result is
// reversed.  Two kernels: a parallel one packs the mask rows to bits and counts degrees; a single work-group then
// walks the levels -- every node's row is scanned exactly once, when the node is in the frontier -- with no host
// round trip and no grid-wide barrier: its loops end when every node has been placed.
#include "bbm_internal.h"

#include <climits>

namespace {

constexpr int kMaxNodes = 65536;            // visited set and one mask row must fit in LDS
constexpr int kOrderThreads = 1024;
constexpr int kPackThreads = 256;
constexpr int kRankChunk = 2048;            // keys of a level staged in LDS at a time
constexpr int kRankPerThread = 4;           // keys a thread ranks per sweep
constexpr int kBatch = 8;                   // row words a thread of the level walk has in flight

// 4 mask bytes -> 4 bits (bit t = byte t non-zero).
__device__ __forceinline__ uint32_t nz_nibble(uint32_t x) {
  uint32_t y = (((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u;
  return (((y >> 7) * 0x00204081u) >> 21) & 0xfu;
}

enum { kStDone = 0, kStLvlLo = 1, kStLvlHi = 2, kStCand = 3, kStInts = 8 };  // state of the level walk (int32)

// One work-group per mask row: bits[row][w] (row-major, bits past N zero), degree[row], parent_pos[row] = "none".
__global__ __launch_bounds__(kPackThreads) void rcm_pack_kernel(const uint8_t* __restrict__ mask, int N, int64_t row_stride, int W,
                                                                uint64_t* __restrict__ bits, int32_t* __restrict__ degree,
                                                                int32_t* __restrict__ parent_pos, uint64_t* __restrict__ visited,
                                                                uint64_t* __restrict__ claimed, int32_t* __restrict__ state) {
  __shared__ int red_s[kPackThreads / 64];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  if (row == 0) {  // the walk's sets (nodes past N count as visited) and state
    for (int w = tid; w < W; w += kPackThreads) {
      visited[w] = (w == W - 1 && (N & 63)) ? ~0ull << (N & 63) : 0ull;
      claimed[w] = 0;
    }
    if (tid < kStInts) state[tid] = 0;
  }
  const uint8_t* __restrict__ src = mask + (int64_t)row * row_stride;
  const bool vec = ((reinterpret_cast<uintptr_t>(mask) | (uintptr_t)row_stride) & 15) == 0;
  int count = 0;
  for (int w = tid; w < W; w += kPackThreads) {
    uint64_t word = 0;
    const int c0 = 64 * w;
    if (vec && c0 + 64 <= N) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint4 x = *reinterpret_cast<const uint4*>(src + c0 + 16 * t);
        const uint64_t b16 = nz_nibble(x.x) | (nz_nibble(x.y) << 4) | (nz_nibble(x.z) << 8) | (nz_nibble(x.w) << 12);
        word |= b16 << (16 * t);
      }
    } else {
      for (int t = 0; t < 64; ++t)
        if (c0 + t < N && src[c0 + t] != 0) word |= 1ull << t;
    }
    bits[(int64_t)row * W + w] = word;
    count += __popcll(word);
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) count += __shfl_xor(count, d);
  if (lane == 0) red_s[tid >> 6] = count;
  __syncthreads();
  if (tid == 0) {
    int total = 0;
    for (int w = 0; w < kPackThreads / 64; ++w) total += red_s[w];
    degree[row] = total;
    parent_pos[row] = INT_MAX;
  }
}

// State of the level walk in the workspace (int32): the walk is cut into kernels -- a fixed number of rounds of a
// parallel expansion (many work-groups) and a one-work-group advance, then a one-work-group finisher that does both
// itself for whatever is left (graphs with more levels or components than rounds).  No kernel waits for another.
constexpr int kRounds = 48;                 // parallel rounds (one breadth-first level, or one component start, each)
constexpr int kExpandWGs = 1024, kExpandThreads = 256;

__device__ __forceinline__ uint64_t level_key(int parent, int degree, int v) {
  return ((uint64_t)(uint32_t)parent << 40) | ((uint64_t)(uint32_t)degree << 20) | (uint64_t)(uint32_t)v;
}

// Ranks the L distinct keys by counting and calls place(rank, node) for each; the keys pass through LDS in chunks and
// a thread ranks up to kRankPerThread keys per sweep.  All kOrderThreads threads of the work-group must call it.
template <typename Place>
__device__ __forceinline__ void rank_level(const uint64_t* keys, int L, uint64_t* chunk_s, int tid, Place place) {
  for (int c0 = 0; c0 < L; c0 += kRankPerThread * kOrderThreads) {
    uint64_t mine[kRankPerThread];
    int r[kRankPerThread];
#pragma unroll
    for (int t = 0; t < kRankPerThread; ++t) {
      const int c = c0 + t * kOrderThreads + tid;
      mine[t] = c < L ? keys[c] : 0;
      r[t] = 0;
    }
    for (int j0 = 0; j0 < L; j0 += kRankChunk) {
      const int n = min(kRankChunk, L - j0);
      __syncthreads();  // the previous chunk has been read
      for (int j = tid; j < n; j += kOrderThreads) chunk_s[j] = keys[j0 + j];
      __syncthreads();
      for (int j = 0; j < n; ++j) {
        const uint64_t kj = chunk_s[j];
#pragma unroll
        for (int t = 0; t < kRankPerThread; ++t) r[t] += kj < mine[t] ? 1 : 0;
      }
    }
#pragma unroll
    for (int t = 0; t < kRankPerThread; ++t)
      if (c0 + t * kOrderThreads + tid < L) place(r[t], (int)(mine[t] & 0xfffffull));
  }
}

// The unvisited node of minimum (degree, index), or -1: every thread of the work-group gets the result.
template <typename Visited>
__device__ __forceinline__ int min_degree_unvisited(const int32_t* __restrict__ degree, int N, Visited visited_word,
                                                    unsigned long long* min_s, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  unsigned long long best = ~0ull;
  for (int i = tid; i < N; i += kOrderThreads)
    if (!((visited_word(i >> 6) >> (i & 63)) & 1ull)) best = min(best, ((unsigned long long)(uint32_t)degree[i] << 32) | (uint32_t)i);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) best = min(best, (unsigned long long)__shfl_xor(best, d));
  __syncthreads();  // min_s may still be read from an earlier call
  if (lane == 0) min_s[wave] = best;
  __syncthreads();
  best = min_s[0];
  for (int w = 1; w < kOrderThreads / 64; ++w) best = min(best, min_s[w]);
  return best == ~0ull ? -1 : (int)(best & 0xffffffffull);
}

// Parallel expansion of the current level: every frontier node's bit row is scanned once; an unvisited neighbour is
// claimed by its earliest parent (atomic minimum of the parent's position) and entered in the candidate list by
// whoever sets its bit in the `claimed` set first.  Returns at once when there is no frontier.
__global__ __launch_bounds__(kExpandThreads) void rcm_expand_kernel(const uint64_t* __restrict__ bits, const int32_t* __restrict__ order,
                                                                    const uint64_t* __restrict__ visited, uint64_t* claimed,
                                                                    int32_t* parent_pos, int32_t* cand, int32_t* state, int W) {
  const int lvl_lo = state[kStLvlLo], lvl_hi = state[kStLvlHi];
  if (state[kStDone] || lvl_lo >= lvl_hi) return;
  const int64_t total = (int64_t)(lvl_hi - lvl_lo) * W;
  const int64_t stride = (int64_t)gridDim.x * kExpandThreads;
  for (int64_t x0 = (int64_t)blockIdx.x * kExpandThreads + threadIdx.x; x0 < total; x0 += kBatch * stride) {
    uint64_t word[kBatch];
    int f[kBatch], w[kBatch];
#pragma unroll
    for (int t = 0; t < kBatch; ++t) {
      const int64_t x = x0 + t * stride;
      word[t] = 0;
      f[t] = w[t] = 0;
      if (x < total) {
        f[t] = lvl_lo + (int)(x / W);
        w[t] = (int)(x % W);
        word[t] = bits[(int64_t)order[f[t]] * W + w[t]] & ~visited[w[t]];
      }
    }
#pragma unroll
    for (int t = 0; t < kBatch; ++t) {
      uint64_t b = word[t];
      while (b) {
        const int v = 64 * w[t] + __builtin_ctzll(b);
        b &= b - 1;
        atomicMin(&parent_pos[v], f[t]);
        const unsigned long long bit = 1ull << (v & 63);
        if (!(atomicOr(reinterpret_cast<unsigned long long*>(&claimed[v >> 6]), bit) & bit)) cand[atomicAdd(&state[kStCand], 1)] = v;
      }
    }
  }
}

// Ranking of the candidates the expansion found (many work-groups): a thread ranks one candidate by counting the
// smaller keys -- every work-group stages all keys of the level through LDS, building them from the candidate list
// as it goes --, places it behind the nodes ordered so far and marks it visited.  Reads the state, changes none of it
// (the advance that follows does).  One work-group ranking a level of 3500 nodes alone takes 0.3 ms.
constexpr int kRankWGs = 256, kRankThreads = 256, kRankStage = 4;  // kRankStage keys of a thread's staging share in flight
__global__ __launch_bounds__(kRankThreads) void rcm_rank_kernel(const int32_t* __restrict__ degree, const int32_t* __restrict__ parent_pos,
                                                                const int32_t* __restrict__ cand, int32_t* __restrict__ order,
                                                                uint64_t* visited, const int32_t* __restrict__ state) {
  __shared__ __attribute__((aligned(16))) uint64_t chunk_s[kRankChunk + 8];
  const int tid = threadIdx.x;
  if (state[kStDone]) return;
  const int n_done = state[kStLvlHi], L = state[kStCand];
  auto key_of = [&](int c) {
    const int v = cand[c];
    return level_key(parent_pos[v], degree[v], v);
  };
  for (int c0 = (int)blockIdx.x * kRankThreads; c0 < L; c0 += (int)gridDim.x * kRankThreads) {  // uniform in the work-group
    const int c = c0 + tid;
    const uint64_t mine = c < L ? key_of(c) : 0;
    int r = 0;
    for (int j0 = 0; j0 < L; j0 += kRankChunk) {
      const int n = min(kRankChunk, L - j0);
      __syncthreads();  // the previous chunk has been read
      for (int j = tid; j < n; j += kRankStage * kRankThreads) {  // a key is three dependent loads: keep several going
        int v[kRankStage], pp[kRankStage], dg[kRankStage];
#pragma unroll
        for (int t = 0; t < kRankStage; ++t) v[t] = j + t * kRankThreads < n ? cand[j0 + j + t * kRankThreads] : 0;
#pragma unroll
        for (int t = 0; t < kRankStage; ++t) {
          pp[t] = parent_pos[v[t]];
          dg[t] = degree[v[t]];
        }
#pragma unroll
        for (int t = 0; t < kRankStage; ++t)
          if (j + t * kRankThreads < n) chunk_s[j + t * kRankThreads] = level_key(pp[t], dg[t], v[t]);
      }
      if (tid < 8) chunk_s[n + tid] = ~0ull;  // pad to a multiple of 8 with keys that count for nobody
      __syncthreads();
      for (int j = 0; j < n; j += 8) {  // 8 keys per LDS round trip
        uint64_t k[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) k[t] = chunk_s[j + t];
#pragma unroll
        for (int t = 0; t < 8; ++t) r += k[t] < mine ? 1 : 0;
      }
    }
    if (c < L) {
      const int v = (int)(mine & 0xfffffull);
      order[n_done + r] = v;
      atomicOr(reinterpret_cast<unsigned long long*>(&visited[v >> 6]), 1ull << (v & 63));
    }
  }
}

// One advance, one work-group: make the candidates the expansion found (ranked and placed by rcm_rank_kernel) the next
// level -- or, when it found none (a component is finished, or nothing has started yet), start the next component.
__global__ __launch_bounds__(kOrderThreads) void rcm_advance_kernel(const int32_t* __restrict__ degree, int32_t* order,
                                                                   uint64_t* visited, int32_t* state, int N) {
  __shared__ unsigned long long min_s[kOrderThreads / 64];
  const int tid = threadIdx.x;
  if (state[kStDone]) return;
  const int n_done = state[kStLvlHi], L = state[kStCand];  // every placed node lies below the end of the current level
  __syncthreads();                                         // everyone has read the state before thread 0 rewrites it
  if (L > 0) {
    if (tid == 0) {
      state[kStLvlLo] = n_done;
      state[kStLvlHi] = n_done + L;
      state[kStCand] = 0;
    }
  } else {
    const int start = min_degree_unvisited(degree, N, [&](int w) { return visited[w]; }, min_s, tid);
    if (tid == 0) {
      if (start < 0) {
        state[kStDone] = 1;
      } else {
        order[n_done] = start;
        visited[start >> 6] |= 1ull << (start & 63);
        state[kStLvlLo] = n_done;
        state[kStLvlHi] = n_done + 1;
      }
    }
  }
}

// The finisher, one work-group: whatever the rounds left (nothing, for graphs of few levels and components) is walked
// here with the expansion done by the same work-group; then the ordering is reversed into perm.  Global arrays written
// by some threads and read by others are separated by an agent-scope fence and a barrier.
__global__ __launch_bounds__(kOrderThreads) void rcm_finish_kernel(const uint64_t* __restrict__ bits, const int32_t* __restrict__ degree,
                                                                   int32_t* parent_pos, int32_t* order, int32_t* cand, uint64_t* keys,
                                                                   const uint64_t* __restrict__ visited_g, const int32_t* __restrict__ state,
                                                                   int N, int W, int32_t* __restrict__ perm) {
  __shared__ uint64_t visited[kMaxNodes / 64];
  __shared__ uint64_t claimed[kMaxNodes / 64];  // nodes some frontier node has reached (they become visited within the level)
  __shared__ uint64_t chunk_s[kRankChunk];
  __shared__ unsigned long long min_s[kOrderThreads / 64];
  __shared__ int count_s;
  const int tid = threadIdx.x;
  auto sync_global = [&]() {
    __threadfence();
    __syncthreads();
  };
  const bool done = state[kStDone] != 0;
  int lvl_lo = state[kStLvlLo], lvl_hi = state[kStLvlHi];
  int n_done = lvl_hi;
  if (!done) {
    for (int w = tid; w < kMaxNodes / 64; w += kOrderThreads) {
      visited[w] = w < W ? visited_g[w] : ~0ull;  // nodes past N were marked visited when the set was initialised
      claimed[w] = 0;
    }
    if (tid == 0) count_s = 0;
    __syncthreads();
    while (true) {
      // ---- breadth-first levels of the current component
      while (lvl_lo < lvl_hi) {
        const int64_t total = (int64_t)(lvl_hi - lvl_lo) * W;
        for (int64_t x0 = tid; x0 < total; x0 += kBatch * kOrderThreads) {
          uint64_t word[kBatch];
          int f[kBatch], w[kBatch];
#pragma unroll
          for (int t = 0; t < kBatch; ++t) {
            const int64_t x = x0 + (int64_t)t * kOrderThreads;
            word[t] = 0;
            f[t] = w[t] = 0;
            if (x < total) {
              f[t] = lvl_lo + (int)(x / W);
              w[t] = (int)(x % W);
              word[t] = bits[(int64_t)order[f[t]] * W + w[t]] & ~visited[w[t]];
            }
          }
#pragma unroll
          for (int t = 0; t < kBatch; ++t) {
            uint64_t b = word[t];
            while (b) {
              const int v = 64 * w[t] + __builtin_ctzll(b);
              b &= b - 1;
              atomicMin(&parent_pos[v], f[t]);  // result unused: a thread's atomics pipeline instead of each waiting for its return
              const unsigned long long bit = 1ull << (v & 63);
              if (!(atomicOr(reinterpret_cast<unsigned long long*>(&claimed[v >> 6]), bit) & bit)) cand[atomicAdd(&count_s, 1)] = v;
            }
          }
        }
        sync_global();
        const int L = count_s;
        for (int c = tid; c < L; c += kOrderThreads) {
          const int v = cand[c];
          keys[c] = level_key(parent_pos[v], degree[v], v);
        }
        sync_global();
        rank_level(keys, L, chunk_s, tid, [&](int r, int v) {
          order[n_done + r] = v;
          atomicOr(reinterpret_cast<unsigned long long*>(&visited[v >> 6]), 1ull << (v & 63));
        });
        if (tid == 0) count_s = 0;
        lvl_lo = lvl_hi;
        lvl_hi = n_done + L;
        n_done += L;
        sync_global();
      }
      // ---- next component
      const int start = min_degree_unvisited(degree, N, [&](int w) { return visited[w]; }, min_s, tid);
      if (start < 0) break;
      if (tid == 0) {
        order[n_done] = start;
        visited[start >> 6] |= 1ull << (start & 63);
      }
      lvl_lo = n_done;
      lvl_hi = n_done + 1;
      n_done += 1;
      sync_global();
    }
  }
  sync_global();
  // the ordering reversed
  for (int k = tid; k < N; k += kOrderThreads) perm[k] = order[N - 1 - k];
}

// out[m][i][j] = mask[m][perm[i]][perm[j]]: one work-group per output row stages the source row in LDS.
__global__ __launch_bounds__(256) void permute_mask_kernel(const uint8_t* __restrict__ mask, int N, int64_t row_stride,
                                                           const int32_t* __restrict__ perm, uint8_t* __restrict__ out) {
  __shared__ __attribute__((aligned(16))) uint8_t row_s[kMaxNodes];
  const int i = blockIdx.x, tid = threadIdx.x;
  const int64_t m = blockIdx.y;
  // entries of perm outside [0, N) are clamped: a wrong permutation gives a wrong mask, never a wild access
  const uint8_t* __restrict__ src = mask + (m * N + min(max(perm[i], 0), N - 1)) * row_stride;
  const bool vec = ((reinterpret_cast<uintptr_t>(mask) | (uintptr_t)row_stride) & 15) == 0;
  if (vec) {
    for (int c = 16 * tid; c < N; c += 16 * 256) {
      if (c + 16 <= N) *reinterpret_cast<uint4*>(row_s + c) = *reinterpret_cast<const uint4*>(src + c);
      else
        for (int t = 0; c + t < N; ++t) row_s[c + t] = src[c + t];
    }
  } else {
    for (int c = tid; c < N; c += 256) row_s[c] = src[c];
  }
  __syncthreads();
  uint8_t* __restrict__ dst = out + (m * N + i) * (int64_t)N;
  if ((N & 15) == 0 && ((reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(perm)) & 15) == 0) {
    // 16 output bytes per lane: four 16-byte reads of perm, sixteen LDS byte reads, one 16-byte store
    for (int j0 = 16 * tid; j0 < N; j0 += 16 * 256) {
      uint32_t w[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int4 p = *reinterpret_cast<const int4*>(perm + j0 + 4 * g);
        const int pp[4] = {p.x, p.y, p.z, p.w};
        w[g] = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) w[g] |= (uint32_t)row_s[min(max(pp[t], 0), N - 1)] << (8 * t);
      }
      *reinterpret_cast<uint4*>(dst + j0) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  } else {
    for (int j = tid; j < N; j += 256) dst[j] = row_s[min(max(perm[j], 0), N - 1)];
  }
}

// Rows of a [BH][N][d] bf16 tensor: gather (out[k] = in[perm[k]]) or scatter (out[perm[k]] = in[k]); 16 bytes per lane.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ in, const int32_t* __restrict__ perm, uint4* __restrict__ out,
                                                          int64_t N, int chunks, int64_t total, int inverse) {
  const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (bh, k, chunk)
  if (x >= total) return;
  const int ch = (int)(x % chunks);
  const int64_t k = (x / chunks) % N, bh = x / chunks / N;
  const int64_t p = min<int64_t>(max(perm[k], 0), N - 1);  // clamped: never a wild access
  const int64_t from = inverse ? k : p, to = inverse ? p : k;
  out[(bh * N + to) * chunks + ch] = in[(bh * N + from) * chunks + ch];
}

inline size_t round256(size_t n) { return (n + 255) / 256 * 256; }
struct RcmLayout {
  size_t bits, degree, parent, order, cand, keys, visited, claimed, state, total;
  explicit RcmLayout(int64_t N) {
    const size_t W = (size_t)((N + 63) / 64);
    size_t o = 0;
    bits = o;
    o += round256((size_t)N * W * 8);
    degree = o;
    o += round256((size_t)N * 4);
    parent = o;
    o += round256((size_t)N * 4);
    order = o;
    o += round256((size_t)N * 4);
    cand = o;
    o += round256((size_t)N * 4);
    keys = o;
    o += round256((size_t)N * 8);
    visited = o;
    o += round256(W * 8);
    claimed = o;
    o += round256(W * 8);
    state = o;
    o += round256(kStInts * 4);
    total = o;
  }
};

}  // namespace

extern "C" __attribute__((visibility("default"))) size_t bbm_rcm_workspace_bytes(int64_t N) {
  if (N < 1 || N > kMaxNodes) return 0;
  return RcmLayout(N).total;
}

extern "C" __attribute__((visibility("default"))) int bbm_rcm_order(const uint8_t* mask, int64_t N, int64_t row_stride_bytes, int32_t* perm,
                                                                   void* workspace, size_t workspace_bytes, void* stream) {
  using namespace bbm;
  clear_error();
  if (!mask || !perm) return fail(BBM_EINVAL, "bbm_rcm_order: mask and perm must not be NULL");
  if (N < 1) return fail(BBM_EINVAL, "bbm_rcm_order: N=%lld must be >= 1", (long long)N);
  if (N > kMaxNodes) return fail(BBM_EUNSUPPORTED, "bbm_rcm_order: N=%lld exceeds %d", (long long)N, kMaxNodes);
  if (row_stride_bytes < N) return fail(BBM_EINVAL, "bbm_rcm_order: row_stride_bytes=%lld < N=%lld", (long long)row_stride_bytes, (long long)N);
  if (!aligned(perm, 4)) return fail(BBM_EINVAL, "bbm_rcm_order: perm must be 4-byte aligned");
  const RcmLayout lay(N);
  if (!workspace || workspace_bytes < lay.total)
    return fail(BBM_EWORKSPACE, "bbm_rcm_order: workspace of %zu bytes needed, %zu given", lay.total, workspace ? workspace_bytes : (size_t)0);
  if (!aligned(workspace, 16)) return fail(BBM_EINVAL, "bbm_rcm_order: workspace must be 16-byte aligned");
  char* ws = static_cast<char*>(workspace);
  uint64_t* bits = reinterpret_cast<uint64_t*>(ws + lay.bits);
  int32_t* degree = reinterpret_cast<int32_t*>(ws + lay.degree);
  int32_t* parent = reinterpret_cast<int32_t*>(ws + lay.parent);
  int32_t* order = reinterpret_cast<int32_t*>(ws + lay.order);
  int32_t* cand = reinterpret_cast<int32_t*>(ws + lay.cand);
  uint64_t* keys = reinterpret_cast<uint64_t*>(ws + lay.keys);
  const int W = (int)ceil_div(N, 64);
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint64_t* visited = reinterpret_cast<uint64_t*>(ws + lay.visited);
  uint64_t* claimed = reinterpret_cast<uint64_t*>(ws + lay.claimed);
  int32_t* state = reinterpret_cast<int32_t*>(ws + lay.state);
  rcm_pack_kernel<<<(unsigned)N, kPackThreads, 0, s>>>(mask, (int)N, row_stride_bytes, W, bits, degree, parent, visited, claimed, state);
  int rc = launch_status("bbm_rcm_order (pack)");
  if (rc != BBM_OK) return rc;
  // the first advance starts the first component; then kRounds rounds of (parallel expansion, ranking, advance); the finisher
  // walks whatever is left and writes perm.  Kernels that find the walk finished return at once.
  rcm_advance_kernel<<<1, kOrderThreads, 0, s>>>(degree, order, visited, state, (int)N);
  for (int r = 0; r < kRounds; ++r) {
    rcm_expand_kernel<<<kExpandWGs, kExpandThreads, 0, s>>>(bits, order, visited, claimed, parent, cand, state, W);
    rcm_rank_kernel<<<kRankWGs, kRankThreads, 0, s>>>(degree, parent, cand, order, visited, state);
    rcm_advance_kernel<<<1, kOrderThreads, 0, s>>>(degree, order, visited, state, (int)N);
  }
  rc = launch_status("bbm_rcm_order (rounds)");
  if (rc != BBM_OK) return rc;
  rcm_finish_kernel<<<1, kOrderThreads, 0, s>>>(bits, degree, parent, order, cand, keys, visited, state, (int)N, W, perm);
  return launch_status("bbm_rcm_order");
}

extern "C" __attribute__((visibility("default"))) int bbm_permute_mask(const uint8_t* mask, int64_t Mb, int64_t N, int64_t row_stride_bytes,
                                                                      const int32_t* perm, uint8_t* out, void* stream) {
  using namespace bbm;
  clear_error();
  if (!mask || !perm || !out) return fail(BBM_EINVAL, "bbm_permute_mask: mask, perm, out must not be NULL");
  if (mask == out) return fail(BBM_EINVAL, "bbm_permute_mask: out must not be the input");
  if (Mb < 1 || N < 1) return fail(BBM_EINVAL, "bbm_permute_mask: Mb=%lld, N=%lld must be >= 1", (long long)Mb, (long long)N);
  if (N > kMaxNodes || Mb > 65535) return fail(BBM_EUNSUPPORTED, "bbm_permute_mask: N=%lld exceeds %d or Mb=%lld exceeds 65535", (long long)N, kMaxNodes, (long long)Mb);
  if (row_stride_bytes < N) return fail(BBM_EINVAL, "bbm_permute_mask: row_stride_bytes=%lld < N=%lld", (long long)row_stride_bytes, (long long)N);
  permute_mask_kernel<<<dim3((unsigned)N, (unsigned)Mb), 256, 0, static_cast<hipStream_t>(stream)>>>(mask, (int)N, row_stride_bytes, perm, out);
  return launch_status("bbm_permute_mask");
}

extern "C" __attribute__((visibility("default"))) int bbm_gather_rows(const void* in, const int32_t* perm, void* out, int64_t BH, int64_t N, int d,
                                                                     int inverse, void* stream) {
  using namespace bbm;
  clear_error();
  if (!in || !perm || !out) return fail(BBM_EINVAL, "bbm_gather_rows: in, perm, out must not be NULL");
  if (in == out) return fail(BBM_EINVAL, "bbm_gather_rows: out must not be the input");
  if (!aligned(in, 16) || !aligned(out, 16)) return fail(BBM_EINVAL, "bbm_gather_rows: in and out must be 16-byte aligned");
  if (BH < 1 || N < 1 || d < 8 || d % 8 != 0) return fail(BBM_EINVAL, "bbm_gather_rows: BH=%lld, N=%lld >= 1 and d=%d a multiple of 8 required", (long long)BH, (long long)N, d);
  const int chunks = d / 8;
  const int64_t total = BH * N * chunks;
  if (ceil_div(total, 256) >= (1ll << 31)) return fail(BBM_EUNSUPPORTED, "bbm_gather_rows: tensor too large");
  gather_rows_kernel<<<(unsigned)ceil_div(total, 256), 256, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const uint4*>(in), perm, static_cast<uint4*>(out), N, chunks, total, inverse ? 1 : 0);
  return launch_status("bbm_gather_rows");
}
