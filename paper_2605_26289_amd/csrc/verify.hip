// Greedy verification of speculative batches on the device (paper Sec. 3.8: batched on-device argmax
// over the vocabulary; Alg. 2: accept the drafts that match, front to back).
//
//   argmax_partial_kernel   one workgroup per (row, 32 KiB chunk of the row): 16-byte loads, eight in
//                           flight per lane, running (max, first index) per lane, wavefront shuffle
//                           reduction, one (value, index) pair per chunk.  HBM bound: every logit is
//                           read exactly once.
//   verify_finish_kernel    one wavefront per slot: folds the chunk pairs of each of its rows, then
//                           finds the first draft that differs from the row's argmax.
//
// Ties go to the lowest token id; a NaN logit counts as +infinity.
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace dk {

namespace {

constexpr int VERIFY_THREADS = 256;
constexpr int VERIFY_UNROLL = 8;
constexpr int VERIFY_CHUNK_BYTES = VERIFY_THREADS * 16 * VERIFY_UNROLL;  // 32 KiB of one row per workgroup

struct Best {
  float v;
  int32_t i;
};

__device__ __forceinline__ float as_key(float x) { return x != x ? INFINITY : x; }

// `a` wins over `b` if it is larger, or equal with the lower index
__device__ __forceinline__ Best better(Best a, Best b) {
  const bool take_b = b.v > a.v || (b.v == a.v && b.i < a.i);
  return take_b ? b : a;
}

__device__ __forceinline__ float elem_to_float(float x) { return x; }
__device__ __forceinline__ float elem_to_float(uint16_t bits) { return __uint_as_float((uint32_t)bits << 16); }

template <typename T>
__global__ __launch_bounds__(VERIFY_THREADS) void argmax_partial_kernel(const T* __restrict__ logits, int64_t row_stride,
                                                                        int64_t vocab, int32_t n_chunks,
                                                                        float* __restrict__ part_val,
                                                                        int32_t* __restrict__ part_idx) {
  constexpr int VEC = 16 / (int)sizeof(T);
  constexpr int64_t CHUNK = (int64_t)VERIFY_THREADS * VEC * VERIFY_UNROLL;
  const int32_t row = blockIdx.y, chunk = blockIdx.x;
  const T* p = logits + (int64_t)row * row_stride;
  const int64_t base = (int64_t)chunk * CHUNK;
  uint4 raw[VERIFY_UNROLL];
  bool full[VERIFY_UNROLL];
#pragma unroll
  for (int u = 0; u < VERIFY_UNROLL; ++u) {
    const int64_t e0 = base + ((int64_t)u * VERIFY_THREADS + threadIdx.x) * VEC;
    full[u] = e0 + VEC <= vocab;
    raw[u] = full[u] ? *(const uint4*)(p + e0) : make_uint4(0, 0, 0, 0);
  }
  Best best{-INFINITY, INT32_MAX};
#pragma unroll
  for (int u = 0; u < VERIFY_UNROLL; ++u) {
    const int64_t e0 = base + ((int64_t)u * VERIFY_THREADS + threadIdx.x) * VEC;
    if (full[u]) {
      const T* lane_vals = (const T*)&raw[u];
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        const float v = as_key(elem_to_float(lane_vals[j]));
        // indices only grow along a lane's walk, so "strictly larger" keeps the first maximum
        if (v > best.v || best.i == INT32_MAX) best = Best{v, (int32_t)(e0 + j)};
      }
    } else {
      for (int64_t e = e0; e < vocab && e < e0 + VEC; ++e) {  // ragged end of the row
        const float v = as_key(elem_to_float(p[e]));
        if (v > best.v || best.i == INT32_MAX) best = Best{v, (int32_t)e};
      }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    Best o{__shfl_xor(best.v, off), __shfl_xor(best.i, off)};
    best = better(best, o);
  }
  __shared__ float sv[VERIFY_THREADS / 64];
  __shared__ int32_t si[VERIFY_THREADS / 64];
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    sv[wave] = best.v;
    si[wave] = best.i;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    Best b{sv[0], si[0]};
#pragma unroll
    for (int w = 1; w < VERIFY_THREADS / 64; ++w) b = better(b, Best{sv[w], si[w]});
    part_val[(int64_t)row * n_chunks + chunk] = b.v;
    part_idx[(int64_t)row * n_chunks + chunk] = b.i;
  }
}

// One wavefront per slot.  Batch rows [r0, r1) of the slot hold [G_last, draft 0, ..., draft k-1].
__global__ __launch_bounds__(64) void verify_finish_kernel(const int32_t* __restrict__ cu_delta,
                                                           const float* __restrict__ part_val,
                                                           const int32_t* __restrict__ part_idx, int32_t n_chunks,
                                                           const int32_t* __restrict__ batch_tokens,
                                                           int32_t* __restrict__ argmax_rows,
                                                           int32_t* __restrict__ n_keep_out,
                                                           int32_t* __restrict__ next_token_out) {
  const int32_t b = blockIdx.x, lane = threadIdx.x;
  const int32_t r0 = cu_delta[b], r1 = cu_delta[b + 1];
  if (r1 <= r0) {
    if (lane == 0) {
      n_keep_out[b] = 0;
      next_token_out[b] = -1;
    }
    return;
  }
  for (int32_t r = r0 + lane; r < r1; r += 64) {
    Best best{part_val[(int64_t)r * n_chunks], part_idx[(int64_t)r * n_chunks]};
    for (int32_t c = 1; c < n_chunks; ++c)
      best = better(best, Best{part_val[(int64_t)r * n_chunks + c], part_idx[(int64_t)r * n_chunks + c]});
    argmax_rows[r] = best.i;
  }
  __syncthreads();
  // first draft s (0-based) whose token differs from what the model says after batch position s
  const int32_t k = r1 - r0 - 1;
  int32_t first_bad = k;
  for (int32_t s = lane; s < k; s += 64)
    if (argmax_rows[r0 + s] != batch_tokens[r0 + 1 + s]) {
      first_bad = s;
      break;  // this lane's later candidates are larger anyway
    }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) first_bad = min(first_bad, __shfl_xor(first_bad, off));
  if (lane == 0) {
    n_keep_out[b] = 1 + first_bad;
    next_token_out[b] = argmax_rows[r0 + first_bad];
  }
}

}  // namespace

int64_t verify_workspace_bytes(int32_t total_rows, int64_t vocab, int32_t dtype) {
  const int64_t elem = dtype == 1 ? 2 : 4;
  const int64_t n_chunks = (vocab * elem + VERIFY_CHUNK_BYTES - 1) / VERIFY_CHUNK_BYTES;
  const int64_t pairs = (int64_t)total_rows * n_chunks;
  return ((pairs * 8 + (int64_t)total_rows * 4 + 255) / 256) * 256 + 256;
}

hipError_t launch_verify_greedy(int32_t n_seqs, int32_t total_rows, const int32_t* cu_delta_dev, const void* logits,
                                int32_t dtype, int64_t vocab, int64_t row_stride, const int32_t* batch_tokens,
                                int32_t* argmax_out, int32_t* n_keep_out, int32_t* next_token_out, void* workspace,
                                hipStream_t stream) {
  if (n_seqs <= 0) return hipSuccess;
  const int64_t elem = dtype == 1 ? 2 : 4;
  const int32_t n_chunks = (int32_t)((vocab * elem + VERIFY_CHUNK_BYTES - 1) / VERIFY_CHUNK_BYTES);
  float* part_val = (float*)workspace;
  int32_t* part_idx = (int32_t*)(part_val + (int64_t)total_rows * n_chunks);
  int32_t* am = argmax_out ? argmax_out : part_idx + (int64_t)total_rows * n_chunks;
  if (total_rows > 0) {
    const dim3 grid((unsigned)n_chunks, (unsigned)total_rows);
    if (dtype == 1)
      argmax_partial_kernel<uint16_t><<<grid, VERIFY_THREADS, 0, stream>>>((const uint16_t*)logits, row_stride, vocab,
                                                                            n_chunks, part_val, part_idx);
    else
      argmax_partial_kernel<float><<<grid, VERIFY_THREADS, 0, stream>>>((const float*)logits, row_stride, vocab,
                                                                         n_chunks, part_val, part_idx);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  verify_finish_kernel<<<dim3((unsigned)n_seqs), 64, 0, stream>>>(cu_delta_dev, part_val, part_idx, n_chunks,
                                                                   batch_tokens, am, n_keep_out, next_token_out);
  return hipGetLastError();
}

}  // namespace dk
