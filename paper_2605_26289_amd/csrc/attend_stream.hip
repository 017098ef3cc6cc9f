// bf16 MFMA delta-prefill attention kernels for gfx950 (head_dim 128).
//
// Both kernels compute, for the packed query rows of one KV head (row r = token r / G, head r % G of
// the group), the transposed products S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16.
// In that orientation a lane owns one query row (column l % 32 of the 32x32 result), so the online
// softmax needs one cross-lane exchange per row block and the probabilities leave the first MFMA in
// exactly the register layout the second one wants as its B operand: P never touches LDS.
//
//   tile kernel    large Delta: a workgroup owns 256 packed rows (4 wavefronts x 64 rows) and all
//                  wavefronts share each 64-key K/V tile through LDS (compute bound, MFMA roofline)
//   stream kernel  small Delta (G*Delta <= 64): every wavefront streams its own slice of the keys
//                  through private LDS stages with no barriers, the four states are merged at the
//                  end (HBM bound)
//
// K/V tiles go HBM -> LDS with global_load_lds_dwordx4 (no VGPR staging).  Rows are 256 B; the 16-byte
// chunks of a row are XOR-swizzled so that the K reads (ds_read_b128, one row per lane) and the V
// reads (ds_read_b64_tr_b16, 4 rows x 16 columns per 16 lanes) are bank-conflict free.
#include <hip/hip_runtime.h>

#include "attend_common.hpp"
#include "kernels.hpp"

namespace dk {
namespace mfma {

template <int MB>
struct RowState {
  f32x16 o[4][MB];  // O^T accumulators: [depth block][row block], unnormalised
  float m[MB];      // running maximum of the scaled scores (log2 units), -inf before the first key
  float l[MB];      // this lane's share of the weight sum (the other half-wave holds the rest)
};

// Q as B operand: lane (row l%32 of block mb, half l/32) holds Q[row][ks*16 + 8*(l/32) .. +7].
template <int MB, int KB>
__device__ __forceinline__ void compute_tile(const char* k_lds, const char* v_lds, const bf16x8 (&qf)[MB][8],
                                             RowState<MB>& st, const int (&limit)[MB], float c, int lane, int cnt,
                                             int pos, bool need_mask) {
  f32x16 s[KB][MB];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][mb][r] = 0.f;

#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    bf16x8 a[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) a[kb] = read_k_frag(k_lds, k_lane_off(lane), kb, ks);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        s[kb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kb], qf[mb][ks], s[kb][mb], 0, 0, 0);
  }

  const int h = lane >> 5;
  if (need_mask) {
    // accumulator r of key block kb is key kb*32 + 8*(r/4) + 4h + r%4 of the tile
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int lim = min(cnt - 1, limit[mb] - pos);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
          if (key > lim) s[kb][mb][r] = -INFINITY;
        }
    }
  }

  bf16x8 pf[MB][2 * KB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][mb][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mn = fmaxf(st.m[mb], mx * c);
    const float ms = (mn == -INFINITY) ? 0.f : mn;  // every key so far masked: keep the arithmetic finite
    const float alpha = __builtin_amdgcn_exp2f(st.m[mb] - ms);
    float rs = 0.f;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][mb][r], c, -ms));
        rs += p;
        s[kb][mb][r] = p;
      }
    st.l[mb] = st.l[mb] * alpha + rs;
    st.m[mb] = mn;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][mb][r] *= alpha;
#pragma unroll
    for (int j = 0; j < 2 * KB; ++j)
#pragma unroll
      for (int t = 0; t < 8; ++t) pf[mb][j][t] = (__bf16)s[j >> 1][mb][8 * (j & 1) + t];
  }

#pragma unroll
  for (int j = 0; j < 2 * KB; ++j) {
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const bf16x8 vf = read_v_frag(v_lds, v_lane_off(lane), j, db);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        st.o[db][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[mb][j], st.o[db][mb], 0, 0, 0);
    }
  }
}

// Accumulator r of depth block db is depth db*32 + 8*(r/4) + 4h + r%4: four consecutive depths per r/4.
// Writes depth block `db` of the wavefront's rows, either as fp32 partial sums or as final bf16 output.
// ------------------------------------------------------------------------------------------------
// Stream kernel.  grid = items * n_kv_heads, block = 256.  Each wavefront owns a quarter of the item's
// key range and two private 32-key stages (K 8 KiB + V 8 KiB each); no barrier in the loop.  At the
// end the four (O, m, l) states are merged through LDS, wavefront w finishing depth block w.
// ------------------------------------------------------------------------------------------------
constexpr int STREAM_KT = 32;
constexpr int STREAM_STAGE_BYTES = 2 * STREAM_KT * ROW_BYTES;  // 16 KiB
constexpr int STREAM_WAVE_BYTES = 2 * STREAM_STAGE_BYTES;      // 32 KiB
constexpr int STREAM_ML_OFFSET = 4 * STREAM_WAVE_BYTES;        // after the stages / the merge buffer
constexpr int STREAM_LDS_BYTES = STREAM_ML_OFFSET + 4 * 64 * 2 * 4;

__global__ __launch_bounds__(256, 1) void attend_stream_kernel(Ctx c) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int MB = 2;
  const int g = blockIdx.x % c.n_kv_heads;
  const DkItem it = load_desc(c.items, blockIdx.x / c.n_kv_heads);
  const DkEntry e = load_desc(c.entries, it.entry);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int last_row = it.row0 + it.nrows - 1;
  const int min_limit = e.n + (it.row0 >> c.gshift);

  bf16x8 qf[MB][8];
  int limit[MB];
  load_q<MB>(c, e, g, it.row0, last_row, lane, qf, limit);

  RowState<MB> st;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    st.m[mb] = -INFINITY;
    st.l[mb] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][mb][r] = 0.f;
  }

  const int ntile = (it.kv_hi - it.kv_lo + STREAM_KT - 1) / STREAM_KT;
  const int per = (ntile + 3) / 4 * STREAM_KT;
  const int lo = min(it.kv_hi, it.kv_lo + wave * per);
  const int hi = min(it.kv_hi, lo + per);
  char* my = smem + wave * STREAM_WAVE_BYTES;

  KvCursor cur{c.segs, e.seg_begin, e.seg_end, lo, hi};
  KvTile tc, tn;
  bool have = cur.next(c, g, STREAM_KT, tc);
  auto issue = [&](const KvTile& t, int stage) {
    char* kl = my + stage * STREAM_STAGE_BYTES;
    char* vl = kl + STREAM_KT * ROW_BYTES;
#pragma unroll
    for (int b = 0; b < 8; ++b) load_rows4<false>(t.k, t.stride, t.cnt, kl, b, lane);
#pragma unroll
    for (int b = 0; b < 8; ++b) load_rows4<true>(t.v, t.stride, t.cnt, vl, b, lane);
  };
  if (have) issue(tc, 0);
  int stage = 0;
  while (have) {
    const bool have_next = cur.next(c, g, STREAM_KT, tn);
    if (have_next) {
      issue(tn, stage ^ 1);
      wait_vmcnt<16>();
    } else {
      wait_vmcnt<0>();
    }
    const char* kl = my + stage * STREAM_STAGE_BYTES;
    const bool need_mask = tc.cnt < STREAM_KT || tc.pos + STREAM_KT - 1 > min_limit;
    compute_tile<MB, 1>(kl, kl + STREAM_KT * ROW_BYTES, qf, st, limit, c.c, lane, tc.cnt, tc.pos, need_mask);
    tc = tn;
    have = have_next;
    stage ^= 1;
  }

  // ---- merge the four wavefront states -------------------------------------------------------
  __syncthreads();  // every wavefront is done with its stages: the space becomes the merge buffer
  float* obuf = (float*)smem;                       // [wave][db][mb][r][lane]
  float* ml = (float*)(smem + STREAM_ML_OFFSET);    // [wave][row 0..63][m, l]
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) obuf[(((wave * 4 + db) * MB + mb) * 16 + r) * 64 + lane] = st.o[db][mb][r];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const float lt = st.l[mb] + __shfl_xor(st.l[mb], 32);
    if (lane < 32) {
      ml[(wave * 64 + mb * 32 + lane) * 2] = st.m[mb];
      ml[(wave * 64 + mb * 32 + lane) * 2 + 1] = lt;
    }
  }
  __syncthreads();
  const int db = wave;
  f32x16 acc[MB];
  float mm[MB], ll[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int row = mb * 32 + (lane & 31);
    float mw[4], lw[4];
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      mw[w] = ml[(w * 64 + row) * 2];
      lw[w] = ml[(w * 64 + row) * 2 + 1];
      mx = fmaxf(mx, mw[w]);
    }
    const float ms = (mx == -INFINITY) ? 0.f : mx;
    float lsum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mb][r] = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = __builtin_amdgcn_exp2f(mw[w] - ms);
      lsum += f * lw[w];
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mb][r] += f * obuf[(((w * 4 + db) * MB + mb) * 16 + r) * 64 + lane];
    }
    mm[mb] = mx;
    ll[mb] = lsum;
  }
  store_block<MB>(c, e, it, g, 0, lane, db, acc, ll);
  if (wave == 0) store_ml<MB>(c, e, it, g, 0, lane, mm, ll);
}

}  // namespace mfma

hipError_t launch_attend_stream(const AttendArgs& a, const DkItem* items, int32_t n_items, hipStream_t stream) {
  using namespace mfma;
  if (n_items <= 0) return hipSuccess;
  if (a.arena.head_dim != D || a.arena.dtype != 1) return hipErrorInvalidValue;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)attend_stream_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       STREAM_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const Ctx c = make_ctx(a, items);
  attend_stream_kernel<<<dim3((unsigned)n_items * a.arena.n_kv_heads), 256, STREAM_LDS_BYTES, stream>>>(c);
  return hipGetLastError();
}

}  // namespace dk
