// KV copy kernels, the scalar reference attention kernel and the split merge kernel (gfx950).
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace dk {

// ---------------------------------------------------------------------------------------------
// kv_append / gather: pure row copies between the token-major staging layout
// [token][kv_head][D] and the head-major arena [kv_head][cell][D].  One thread moves 16 bytes.
// Paper Alg. 1: the cache write inside Decode(sigma, batch); only the delta cells are written.
// ---------------------------------------------------------------------------------------------
template <bool TO_ARENA>
__global__ __launch_bounds__(256) void kv_copy_kernel(uint4* __restrict__ k_arena, uint4* __restrict__ v_arena,
                                                      uint4* __restrict__ k_tok, uint4* __restrict__ v_tok,
                                                      const int32_t* __restrict__ cell_of, int64_t tok_base,
                                                      int32_t n_tok, int32_t n_kv_heads, int32_t row_vec,
                                                      int64_t arena_cells) {
  const int64_t per_tok = (int64_t)n_kv_heads * row_vec;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= per_tok * n_tok) return;
  const int32_t t = (int32_t)(idx / per_tok);
  const int32_t rem = (int32_t)(idx - (int64_t)t * per_tok);
  const int32_t g = rem / row_vec;
  const int32_t c = rem - g * row_vec;
  const int64_t cell = cell_of[t];
  if (cell < 0) return;
  const int64_t tok_off = ((tok_base + t) * n_kv_heads + g) * row_vec + c;
  const int64_t arena_off = ((int64_t)g * arena_cells + cell) * row_vec + c;
  uint4* arena = blockIdx.y ? v_arena : k_arena;
  uint4* tok = blockIdx.y ? v_tok : k_tok;
  if (TO_ARENA) arena[arena_off] = tok[tok_off];
  else tok[tok_off] = arena[arena_off];
}

static int32_t row_vecs(const ArenaView& a) { return a.head_dim * (a.dtype == 0 ? 4 : 2) / 16; }

// Short appends (a verify step, a tool result of a few hundred tokens): the destination cells travel
// inside the kernel arguments, so no table has to be copied to the device before the launch -- on a
// short turn that copy and the dependency bubble after it cost more than the append itself.
struct InlineCells {
  int32_t cell[KV_INLINE_MAX_TOKENS];
};
static_assert(sizeof(InlineCells) + 128 <= 4096, "kernel arguments are limited to 4 KiB");

__global__ __launch_bounds__(256) void kv_scatter_inline_kernel(InlineCells cells, uint4* __restrict__ k_arena,
                                                                uint4* __restrict__ v_arena,
                                                                const uint4* __restrict__ k_tok,
                                                                const uint4* __restrict__ v_tok, int32_t n_tok,
                                                                int32_t n_kv_heads, int32_t row_vec,
                                                                int64_t arena_cells) {
  // `cells` is the first argument: it starts the kernel-argument segment.  Reading it through the
  // segment pointer keeps the (lane-dependent) index from forcing a private copy of the whole table.
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const_i32_ptr cell_of = (const_i32_ptr)__builtin_amdgcn_kernarg_segment_ptr();
  (void)cells;
  const int32_t per_tok = n_kv_heads * row_vec;
  const int32_t idx = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
  if (idx >= per_tok * n_tok) return;
  const int32_t t = idx / per_tok;
  const int32_t rem = idx - t * per_tok;
  const int32_t g = rem / row_vec;
  const int32_t c = rem - g * row_vec;
  const int64_t cell = cell_of[t];
  if (cell < 0) return;
  const int64_t tok_off = ((int64_t)t * n_kv_heads + g) * row_vec + c;
  const int64_t arena_off = ((int64_t)g * arena_cells + cell) * row_vec + c;
  if (blockIdx.y) v_arena[arena_off] = v_tok[tok_off];
  else k_arena[arena_off] = k_tok[tok_off];
}

hipError_t launch_kv_scatter_inline(const ArenaView& a, void* k_arena, void* v_arena, const int64_t* cell_of_host,
                                    int32_t n_tok, const void* k_new, const void* v_new, hipStream_t stream) {
  if (n_tok <= 0) return hipSuccess;
  if (n_tok > KV_INLINE_MAX_TOKENS) return hipErrorInvalidValue;
  InlineCells cells{};
  for (int32_t t = 0; t < n_tok; ++t) cells.cell[t] = (int32_t)cell_of_host[t];
  const int32_t rv = row_vecs(a);
  const int64_t work = (int64_t)n_tok * a.n_kv_heads * rv;
  dim3 grid((unsigned)((work + 255) / 256), 2);
  kv_scatter_inline_kernel<<<grid, 256, 0, stream>>>(cells, (uint4*)k_arena, (uint4*)v_arena, (const uint4*)k_new,
                                                     (const uint4*)v_new, n_tok, a.n_kv_heads, rv, a.arena_cells);
  return hipGetLastError();
}

hipError_t launch_kv_scatter(const ArenaView& a, void* k_arena, void* v_arena, const int32_t* cell_of_dev,
                             int64_t tok_base, int32_t n_tok, const void* k_new, const void* v_new,
                             hipStream_t stream) {
  if (n_tok <= 0) return hipSuccess;
  const int32_t rv = row_vecs(a);
  const int64_t work = (int64_t)n_tok * a.n_kv_heads * rv;
  dim3 grid((unsigned)((work + 255) / 256), 2);
  kv_copy_kernel<true><<<grid, 256, 0, stream>>>((uint4*)k_arena, (uint4*)v_arena, (uint4*)k_new, (uint4*)v_new,
                                                 cell_of_dev, tok_base, n_tok, a.n_kv_heads, rv, a.arena_cells);
  return hipGetLastError();
}

hipError_t launch_kv_gather(const ArenaView& a, const int32_t* cell_of_dev, int64_t tok_base, int32_t n_tok,
                            void* k_out, void* v_out, hipStream_t stream) {
  if (n_tok <= 0) return hipSuccess;
  const int32_t rv = row_vecs(a);
  const int64_t work = (int64_t)n_tok * a.n_kv_heads * rv;
  dim3 grid((unsigned)((work + 255) / 256), 2);
  kv_copy_kernel<false><<<grid, 256, 0, stream>>>((uint4*)a.k_arena, (uint4*)a.v_arena, (uint4*)k_out, (uint4*)v_out,
                                                  cell_of_dev, tok_base, n_tok, a.n_kv_heads, rv, a.arena_cells);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Reference attention kernel.  One wavefront per (new token i, query head h).  Each lane walks
// the visible keys lane, lane+64, ... of every segment with its own online-softmax state; the 64
// states are merged through LDS at the end.  Used for fp32 pools, for shapes the MFMA kernels do
// not cover, and as a second GPU implementation in the tests.
// Row i of an entry sees positions 0 .. n+i (bottom-right causal alignment).
// ---------------------------------------------------------------------------------------------
__device__ inline float to_float(float x) { return x; }
__device__ inline float to_float(__bf16 x) { return (float)x; }
__device__ inline void store_out(float* p, float x) { *p = x; }
__device__ inline void store_out(__bf16* p, float x) { *p = (__bf16)x; }

// 16-byte row loads, widened to float
template <typename T> struct VEC;
template <> struct VEC<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float* f) {
    const float4 v = *(const float4*)p;
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
};
template <> struct VEC<__bf16> {
  static constexpr int N = 8;
  __device__ static void load(const __bf16* p, float* f) {
    const uint4 v = *(const uint4*)p;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      f[2 * u] = __uint_as_float(w[u] << 16);
      f[2 * u + 1] = __uint_as_float(w[u] & 0xffff0000u);
    }
  }
};

// The first argument of the attention kernels: the descriptor blob itself when it is small enough to travel in
// the kernel arguments (descriptor pointers are then byte offsets from the start of the argument segment).
template <bool INLINE> struct BlobParam;
template <> struct BlobParam<true> { InlineBlob blob; };
template <> struct BlobParam<false> { char unused; };
template <bool INLINE, typename P>
__device__ __forceinline__ const P* from_blob(const P* p) {
  if constexpr (INLINE) {
    typedef const __attribute__((address_space(4))) char* const_char_ptr;
    return (const P*)((uintptr_t)(const_char_ptr)__builtin_amdgcn_kernarg_segment_ptr() + (uintptr_t)p);
  } else {
    return p;
  }
}

template <typename T, int D, bool INLINE>
__global__ __launch_bounds__(64) void attend_ref_kernel(BlobParam<INLINE> blob, const DkEntry* entries, int32_t n_entries,
                                                        const DkSeg* segs, const T* __restrict__ q,
                                                        const T* __restrict__ k_arena, const T* __restrict__ v_arena,
                                                        const T* __restrict__ k_new, const T* __restrict__ v_new,
                                                        T* __restrict__ out, float* __restrict__ lse, float scale,
                                                        int32_t n_q_heads, int32_t n_kv_heads, int64_t arena_cells) {
  __shared__ float qs[D];
  __shared__ float red[64][D + 1];
  (void)blob;
  entries = from_blob<INLINE>(entries);
  segs = from_blob<INLINE>(segs);
  const int lane = threadIdx.x;
  const int tok = blockIdx.x / n_q_heads;
  const int h = blockIdx.x - tok * n_q_heads;
  // entry that owns this token: entries are ordered by tok0; those with delta == 0 own nothing
  int lo = 0, hi = n_entries - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (entries[mid].tok0 <= tok) lo = mid; else hi = mid - 1;
  }
  while (entries[lo].delta == 0 || tok >= entries[lo].tok0 + entries[lo].delta) --lo;  // skip empty entries sharing tok0
  const DkEntry e = entries[lo];
  const int i = tok - e.tok0;
  const int visible = e.n + i + 1;
  const int g = h / (n_q_heads / n_kv_heads);
  const float s2 = scale * 1.4426950408889634f;  // scores kept in log2 units

  for (int d = lane; d < D; d += 64) qs[d] = to_float(q[((int64_t)tok * n_q_heads + h) * D + d]) * s2;
  __syncthreads();

  float m = -INFINITY, l = 0.f;
  float o[D];
#pragma unroll
  for (int d = 0; d < D; ++d) o[d] = 0.f;

  for (int si = e.seg_begin; si < e.seg_end; ++si) {
    const DkSeg sg = segs[si];
    if (sg.pos >= visible) break;
    const int cnt = min(sg.len, visible - sg.pos);
    for (int j = lane; j < cnt; j += 64) {
      const T *kr, *vr;
      if (sg.src == 0) {
        const int64_t off = ((int64_t)g * arena_cells + sg.start + j) * D;
        kr = k_arena + off;
        vr = v_arena + off;
      } else {
        const int64_t off = ((sg.start + j) * n_kv_heads + g) * D;
        kr = k_new + off;
        vr = v_new + off;
      }
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < D / VEC<T>::N; ++c) {
        float kf[VEC<T>::N];
        VEC<T>::load(kr + c * VEC<T>::N, kf);
#pragma unroll
        for (int u = 0; u < VEC<T>::N; ++u) s += qs[c * VEC<T>::N + u] * kf[u];
      }
      const float mn = fmaxf(m, s);
      const float alpha = exp2f(m - mn);  // m == -inf on the first key: exp2(-inf) == 0
      const float p = exp2f(s - mn);
      l = l * alpha + p;
#pragma unroll
      for (int c = 0; c < D / VEC<T>::N; ++c) {
        float vf[VEC<T>::N];
        VEC<T>::load(vr + c * VEC<T>::N, vf);
#pragma unroll
        for (int u = 0; u < VEC<T>::N; ++u) o[c * VEC<T>::N + u] = o[c * VEC<T>::N + u] * alpha + p * vf[u];
      }
      m = mn;
    }
  }
  // merge the 64 lane states
  float mw = m;
  for (int off = 32; off; off >>= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
  const float f = (m == -INFINITY) ? 0.f : exp2f(m - mw);
  float lw = l * f;
  for (int off = 32; off; off >>= 1) lw += __shfl_xor(lw, off);
#pragma unroll
  for (int d = 0; d < D; ++d) red[lane][d] = o[d] * f;
  __syncthreads();
  const float inv = 1.f / lw;
  for (int d = lane; d < D; d += 64) {
    float acc = 0.f;
    for (int r = 0; r < 64; ++r) acc += red[r][d];
    store_out(&out[((int64_t)tok * n_q_heads + h) * D + d], acc * inv);
  }
  if (lse && lane == 0) lse[(int64_t)tok * n_q_heads + h] = (mw + log2f(lw)) * 0.6931471805599453f;
}

hipError_t launch_attend_ref(const AttendArgs& a, hipStream_t stream) {
  if (a.total_tokens <= 0) return hipSuccess;
  const ArenaView& v = a.arena;
  dim3 grid((unsigned)((int64_t)a.total_tokens * v.n_q_heads));
#define DK_REF(T, D)                                                                                            \
  do {                                                                                                          \
    if (a.inline_blob)                                                                                          \
      attend_ref_kernel<T, D, true><<<grid, 64, 0, stream>>>(                                                   \
          BlobParam<true>{*a.inline_blob}, a.entries, a.n_entries, a.segs, (const T*)a.q, (const T*)v.k_arena,  \
          (const T*)v.v_arena, (const T*)a.k_new, (const T*)a.v_new, (T*)a.out, a.lse, a.scale, v.n_q_heads,    \
          v.n_kv_heads, v.arena_cells);                                                                         \
    else                                                                                                        \
      attend_ref_kernel<T, D, false><<<grid, 64, 0, stream>>>(                                                  \
          BlobParam<false>{0}, a.entries, a.n_entries, a.segs, (const T*)a.q, (const T*)v.k_arena,              \
          (const T*)v.v_arena, (const T*)a.k_new, (const T*)a.v_new, (T*)a.out, a.lse, a.scale, v.n_q_heads,    \
          v.n_kv_heads, v.arena_cells);                                                                         \
  } while (0)
  if (v.dtype == 0 && v.head_dim == 64) DK_REF(float, 64);
  else if (v.dtype == 0 && v.head_dim == 128) DK_REF(float, 128);
  else if (v.dtype == 1 && v.head_dim == 64) DK_REF(__bf16, 64);
  else if (v.dtype == 1 && v.head_dim == 128) DK_REF(__bf16, 128);
  else return hipErrorInvalidValue;
#undef DK_REF
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Merge of split key ranges.  Each split left, per (row, KV head), D unnormalised fp32 sums (parts) and its
// running maximum m (log2 units) with its weight sum l (parts_ml).
//   O = sum_s 2^(m_s-M) o_s / sum_s 2^(m_s-M) l_s.
// A wavefront merges MERGE_ROWS rows of one KV head at a time: for each row every lane first takes one split
// and fetches its (m, l), which gives the common maximum, the weights and the weight sum in one round trip;
// then the lanes cover D and add the splits' sums, the loads of all the rows and of two splits in flight
// together.  (One row per wavefront left most of a launch's time to workgroup turnover when rows are split
// only two or three ways.)
// ---------------------------------------------------------------------------------------------
constexpr int MERGE_ROWS = 4;  // rows per wavefront; a workgroup of four wavefronts covers 16 rows

template <int D, bool INLINE>
__global__ __launch_bounds__(256) void attend_merge_kernel(BlobParam<INLINE> blob, const DkMerge* merges,
                                                           const DkEntry* entries,
                                                           const float* __restrict__ parts,
                                                           const float* __restrict__ parts_ml, __bf16* __restrict__ out,
                                                           float* __restrict__ lse, int32_t n_q_heads,
                                                           int32_t n_kv_heads) {
  static_assert(D == 128, "two floats per lane");
  (void)blob;
  merges = from_blob<INLINE>(merges);
  entries = from_blob<INLINE>(entries);
  const DkMerge mg = merges[blockIdx.x];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int r0 = (blockIdx.z * 4 + wave) * MERGE_ROWS;
  if (r0 >= mg.nrows) return;
  const DkEntry e = entries[mg.entry];
  const int g = blockIdx.y;
  const int group = n_q_heads / n_kv_heads;
  const int64_t srow = (int64_t)mg.nrows * n_kv_heads;  // partial rows from one split of a row to the next
  const int64_t stride = srow * D;

  const float* p0[MERGE_ROWS];
  const float* ml0[MERGE_ROWS];
  bool live[MERGE_ROWS];
#pragma unroll
  for (int i = 0; i < MERGE_ROWS; ++i) {
    live[i] = r0 + i < mg.nrows;
    const int64_t prow = (int64_t)(mg.part_row0 + (live[i] ? r0 + i : r0)) * n_kv_heads + g;
    p0[i] = parts + prow * D + lane * 2;
    ml0[i] = parts_ml + prow * 2;
  }

  float2 acc[MERGE_ROWS];
  float lsum[MERGE_ROWS], mmax[MERGE_ROWS];
#pragma unroll
  for (int i = 0; i < MERGE_ROWS; ++i) {
    acc[i] = make_float2(0.f, 0.f);
    lsum[i] = 0.f;
    float m = -INFINITY;
    for (int s = lane; s < mg.nsplit; s += 64) m = fmaxf(m, ml0[i][s * srow * 2]);
    mmax[i] = m;
  }
#pragma unroll
  for (int off = 32; off; off >>= 1)
#pragma unroll
    for (int i = 0; i < MERGE_ROWS; ++i) mmax[i] = fmaxf(mmax[i], __shfl_xor(mmax[i], off));

  for (int s0 = 0; s0 < mg.nsplit; s0 += 64) {
    const int mine = s0 + lane;
    float w_mine[MERGE_ROWS];
#pragma unroll
    for (int i = 0; i < MERGE_ROWS; ++i) {
      w_mine[i] = 0.f;
      if (mine < mg.nsplit) {
        const float2 ml = *(const float2*)(ml0[i] + mine * srow * 2);  // second touch: served from cache
        w_mine[i] = (ml.x == -INFINITY) ? 0.f : exp2f(ml.x - mmax[i]);
        lsum[i] += w_mine[i] * ml.y;
      }
    }
    const int cnt = min(64, mg.nsplit - s0);
    int s = 0;
    for (; s + 2 <= cnt; s += 2) {
      float2 v0[MERGE_ROWS], v1[MERGE_ROWS];
#pragma unroll
      for (int i = 0; i < MERGE_ROWS; ++i) {
        v0[i] = *(const float2*)(p0[i] + (s0 + s) * stride);
        v1[i] = *(const float2*)(p0[i] + (s0 + s + 1) * stride);
      }
#pragma unroll
      for (int i = 0; i < MERGE_ROWS; ++i) {
        const float w0 = __shfl(w_mine[i], s), w1 = __shfl(w_mine[i], s + 1);
        acc[i].x += w0 * v0[i].x + w1 * v1[i].x;
        acc[i].y += w0 * v0[i].y + w1 * v1[i].y;
      }
    }
    if (s < cnt) {
#pragma unroll
      for (int i = 0; i < MERGE_ROWS; ++i) {
        const float2 v = *(const float2*)(p0[i] + (s0 + s) * stride);
        const float w = __shfl(w_mine[i], s);
        acc[i].x += w * v.x;
        acc[i].y += w * v.y;
      }
    }
  }
#pragma unroll
  for (int off = 32; off; off >>= 1)
#pragma unroll
    for (int i = 0; i < MERGE_ROWS; ++i) lsum[i] += __shfl_xor(lsum[i], off);

#pragma unroll
  for (int i = 0; i < MERGE_ROWS; ++i) {
    if (!live[i]) continue;
    const int row = mg.row0 + r0 + i;
    const int tok = e.tok0 + row / group;
    const int h = g * group + row % group;
    const float inv = 1.f / lsum[i];
    __bf16* o = out + ((int64_t)tok * n_q_heads + h) * D + lane * 2;
    o[0] = (__bf16)(acc[i].x * inv);
    o[1] = (__bf16)(acc[i].y * inv);
    if (lse && lane == 0) lse[(int64_t)tok * n_q_heads + h] = (mmax[i] + log2f(lsum[i])) * 0.6931471805599453f;
  }
}

hipError_t launch_attend_merge(const AttendArgs& a, const DkMerge* merges, int32_t n_merges, int32_t max_rows,
                               hipStream_t stream) {
  if (n_merges <= 0) return hipSuccess;
  if (a.arena.head_dim != 128 || max_rows <= 0) return hipErrorInvalidValue;
  const int rows_per_block = 4 * MERGE_ROWS;
  dim3 grid((unsigned)n_merges, (unsigned)a.arena.n_kv_heads, (unsigned)((max_rows + rows_per_block - 1) / rows_per_block));
  if (a.inline_blob)
    attend_merge_kernel<128, true><<<grid, 256, 0, stream>>>(BlobParam<true>{*a.inline_blob}, merges, a.entries, a.parts,
                                                             a.parts_ml, (__bf16*)a.out, a.lse, a.arena.n_q_heads,
                                                             a.arena.n_kv_heads);
  else
    attend_merge_kernel<128, false><<<grid, 256, 0, stream>>>(BlobParam<false>{0}, merges, a.entries, a.parts,
                                                              a.parts_ml, (__bf16*)a.out, a.lse, a.arena.n_q_heads,
                                                              a.arena.n_kv_heads);
  return hipGetLastError();
}

}  // namespace dk
