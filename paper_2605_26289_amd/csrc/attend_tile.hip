// bf16 MFMA delta-prefill attention, large-Delta ("tile") kernel for gfx950, head_dim 128.
//
// A workgroup owns 256 packed query rows of one KV head (4 wavefronts x 64 rows, row r = token r / G,
// head r % G of the group) and walks the visible keys in 64-key tiles that all four wavefronts share
// through a 4-stage LDS ring (HBM -> LDS by global_load_lds_dwordx4, one barrier per tile).
//
// Per tile and wavefront there are 64 MFMAs (32 for S^T = K Q^T, 32 for O^T += V^T P^T, all
// v_mfma_f32_32x32x16_bf16) and 64 score elements per lane for the softmax, whose v_exp_f32 alone
// costs about half the MFMA time.  With one wavefront per SIMD nothing else can hide that VALU work,
// so the loop is software pipelined by hand: while the matrix pipe computes S^T of tile t+1 and then
// PV of tile t, the VALU turns S^T of tile t into P, one or two elements after every MFMA.
//
// Register plan (one wavefront per SIMD, 512 registers): AGPRs hold the O^T accumulators (128) and Q
// (64, read by the MFMAs as B operand straight from AGPRs); VGPRs hold two S^T buffers (2 x 64, the
// MFMAs write them directly, the VALU works on them in place), P (32) and the K/V operand fragments.
// The MFMAs are issued from inline assembly so that this placement is exactly what the compiler
// allocates; the consequence is that MFMA-result hazards are handled by hand (see settle()).
#include <hip/hip_runtime.h>

#include <utility>

#include "attend_common.hpp"
#include "kernels.hpp"

namespace dk {
namespace mfma {

constexpr int TILE_KT = 64;
constexpr int TILE_STAGES = 4;
constexpr int TILE_STAGE_BYTES = 2 * TILE_KT * ROW_BYTES;  // K 16 KiB + V 16 KiB
constexpr int TILE_LDS_BYTES = TILE_STAGES * TILE_STAGE_BYTES;
constexpr int MB = 2;  // 32-row blocks per wavefront

// S^T accumulators live in VGPRs, O^T accumulators and Q in AGPRs.
#ifdef DK_TILE_BUILTIN_MFMA  // diagnosis build: let the compiler place and guard the MFMAs
__device__ __forceinline__ void mfma_s_first(f32x16& s, const bf16x8& k, const bf16x8& q) {
  f32x16 z = {0};
  s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k, q, z, 0, 0, 0);
}
__device__ __forceinline__ void mfma_s(f32x16& s, const bf16x8& k, const bf16x8& q) {
  s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k, q, s, 0, 0, 0);
}
__device__ __forceinline__ void mfma_o(f32x16& o, const bf16x8& v, const bf16x8& p) {
  o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v, p, o, 0, 0, 0);
}
#else
__device__ __forceinline__ void mfma_s_first(f32x16& s, const bf16x8& k, const bf16x8& q) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(k), "a"(q));
}
__device__ __forceinline__ void mfma_s(f32x16& s, const bf16x8& k, const bf16x8& q) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(k), "a"(q));
}
__device__ __forceinline__ void mfma_o(f32x16& o, const bf16x8& v, const bf16x8& p) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o) : "v"(v), "v"(p));
}
#endif

// The compiler does not see that these registers come out of the matrix pipeline, so it would not
// insert the wait states a plain VALU read of a fresh MFMA result needs.  Every place where such a
// read can follow an MFMA closely passes the registers through this first.
__device__ __forceinline__ void settle(f32x16& a, f32x16& b, f32x16& c, f32x16& d) {
  asm volatile("s_nop 15\n\ts_nop 7" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}
__device__ __forceinline__ void settle_acc(f32x16& a) { asm volatile("s_nop 15\n\ts_nop 7" : "+a"(a)); }

// The reference maximum of a row only moves when its maximum grew by more than this (log2 units):
// after the first tiles the rescale of O is rare, and the weights stay below 2^8.
constexpr float RESCALE_SLACK = 8.f;

struct WaveState {
  f32x16 o[4][MB];  // [depth block][row block], AGPR
  float m[MB];      // reference maximum of the scaled scores (log2 units), -inf before the first key
  float l[MB];      // this lane's share of the weight sum
};

// Keys the row may not see (beyond the causal limit or past the end of a ragged tile) get -inf.
// Accumulator r of key block kb is key kb*32 + 8*(r/4) + 4h + r%4 of the tile.
__device__ __forceinline__ void mask_tile(f32x16 (&s)[2][MB], const int (&limit)[MB], int lane, int cnt, int pos) {
  const int h = lane >> 5;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    // key > lim  <=>  (lim - 4h) - (key - 4h) < 0; done with integer sign arithmetic so that the 64
    // decisions do not each occupy a scalar register pair
    const int base = min(cnt - 1, limit[mb] - pos) - 4 * h;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rest = kb * 32 + 8 * (r >> 2) + (r & 3);
        const uint32_t hide = (uint32_t)((base - rest) >> 31);  // all ones if the key is hidden
        const uint32_t bits = __float_as_uint(s[kb][mb][r]);
        s[kb][mb][r] = __uint_as_float((bits & ~hide) | (0xff800000u & hide));
      }
  }
}

// Row maxima of the tile; raises the reference maxima (and rescales O, l) if some row needs it.
__device__ __forceinline__ void update_reference(const f32x16 (&s)[2][MB], WaveState& st, float c) {
  float mx[MB];
  bool grow = false;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    float v = fmaxf(s[0][mb][0], s[1][mb][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) v = fmaxf(v, fmaxf(s[0][mb][r], s[1][mb][r]));
    v = fmaxf(v, __shfl_xor(v, 32));
    mx[mb] = v * c;
    grow |= mx[mb] > st.m[mb] + RESCALE_SLACK;
  }
  if (__builtin_amdgcn_ballot_w64(grow) == 0) return;
  // rare path; settle_acc() pads both the read after the last MFMA and the next MFMA after the write
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const float mn = fmaxf(st.m[mb], mx[mb]);
    const float ms = (mn == -INFINITY) ? 0.f : mn;
    const float alpha = __builtin_amdgcn_exp2f(st.m[mb] - ms);  // 1 for rows whose maximum did not move
    st.m[mb] = mn;
    st.l[mb] *= alpha;
    // whole-register arithmetic only: element-wise inserts into the accumulator tuples make the compiler
    // shuttle all of O between the two register files on every trip of the key loop
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      settle_acc(st.o[db][mb]);
      f32x16 t = st.o[db][mb];
      t = t * alpha;
      st.o[db][mb] = t;
      settle_acc(st.o[db][mb]);
    }
  }
}

// One pipeline step.  sc holds S^T of the current tile (complete), sn receives S^T of the next tile and
// is moved into sc during the last eight MFMAs, when the VALU has nothing else to do (the step body
// exists once in the program, so the two buffers cannot simply trade names).  On a wavefront's last
// tile the next S^T is computed from whatever the next stage holds and never looked at.
//   MFMA  0..31  S^T(next): depth step i/4, key block (i/2)%2, row block i%2
//   MFMA 32..63  PV(current): key step j = (i-32)/8, depth block ((i-32)/2)%4, row block i%2
// Softmax elements are processed in the order PV consumes them, group g = (j, mb) of 8 elements:
// one element after each of MFMAs 0..47, two after each of 48..55, so that group (j, mb) is packed
// to bf16 before MFMA 32 + 8j starts.
struct Step {
  const char* k_next;
  const char* v_cur;
  const bf16x8 (&qf)[MB][8];
  f32x16 (&sc)[2][MB];
  f32x16 (&sn)[2][MB];
  WaveState& st;
  float c;
  uint32_t koff, voff;
  float ms[MB], rs[MB];
  bf16x8 pf[MB][4];
  bf16x8 kf[2][2];  // [depth-step parity][key block]
  bf16x8 vf[2];     // [parity of the (j, db) pair]

  // softmax element E (0..63), in the order PV consumes them
  template <int E>
  __device__ __forceinline__ void element() {
    constexpr int grp = E >> 3, t = E & 7;
    constexpr int mb = grp & 1, j = grp >> 1;
    constexpr int kb = j >> 1, r = 8 * (j & 1) + t;
    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kb][mb][r], c, -ms[mb]));
    rs[mb] += p;
    pf[mb][j][t] = (__bf16)p;
  }

  // MFMA slot I (0..63) with the VALU work that rides along
  template <int I>
  __device__ __forceinline__ void slot() {
    if constexpr (I < 32) {
      constexpr int ks = I >> 2, kb = (I >> 1) & 1, mb = I & 1;
      if constexpr ((I & 3) == 0 && ks + 1 < 8) {
        kf[(ks + 1) & 1][0] = read_k_frag(k_next, koff, 0, ks + 1);
        kf[(ks + 1) & 1][1] = read_k_frag(k_next, koff, 1, ks + 1);
      }
      if constexpr (ks == 0) mfma_s_first(sn[kb][mb], kf[0][kb], qf[mb][0]);
      else mfma_s(sn[kb][mb], kf[ks & 1][kb], qf[mb][ks]);
      if constexpr (I == 28) vf[0] = read_v_frag(v_cur, voff, 0, 0);
    } else {
      constexpr int pair = (I - 32) >> 1, mb = I & 1;  // pair = j * 4 + db
      constexpr int j = pair >> 2, db = pair & 3;
      if constexpr (mb == 0 && pair + 1 < 16)
        vf[(pair + 1) & 1] = read_v_frag(v_cur, voff, (pair + 1) >> 2, (pair + 1) & 3);
      mfma_o(st.o[db][mb], vf[pair & 1], pf[mb][j]);
    }
    if constexpr (I < 48) {
      element<I>();
    } else if constexpr (I < 56) {
      element<48 + 2 * (I - 48)>();
      element<48 + 2 * (I - 48) + 1>();
    } else {
      // 8 of the 64 registers of the next S^T per slot: [kb][mb] block (I-56)/2, half (I-56)%2
      constexpr int blk = (I - 56) >> 1, half = (I - 56) & 1;
#pragma unroll
      for (int r = 0; r < 8; ++r) sc[blk >> 1][blk & 1][8 * half + r] = sn[blk >> 1][blk & 1][8 * half + r];
    }
    __builtin_amdgcn_sched_barrier(0);
  }

  template <int... Is>
  __device__ __forceinline__ void run(std::integer_sequence<int, Is...>) {
    (slot<Is>(), ...);
  }
};

__device__ __forceinline__ void tile_step(const char* k_next, const char* v_cur, const bf16x8 (&qf)[MB][8],
                                          f32x16 (&sc)[2][MB], f32x16 (&sn)[2][MB], WaveState& st,
                                          const int (&limit)[MB], float c, int lane, int cnt, int pos,
                                          bool need_mask, uint32_t koff, uint32_t voff) {
  Step s{k_next, v_cur, qf, sc, sn, st, c, koff, voff};
  s.kf[0][0] = read_k_frag(k_next, koff, 0, 0);
  s.kf[0][1] = read_k_frag(k_next, koff, 1, 0);
  if (need_mask) mask_tile(sc, limit, lane, cnt, pos);
  update_reference(sc, st, c);
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    s.ms[mb] = (st.m[mb] == -INFINITY) ? 0.f : st.m[mb];
    s.rs[mb] = 0.f;
  }
  __builtin_amdgcn_sched_barrier(0);
  s.run(std::make_integer_sequence<int, 64>{});
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) st.l[mb] += s.rs[mb];
}

__global__ __launch_bounds__(256, 1) void attend_tile_kernel(Ctx c) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int g = blockIdx.x % c.n_kv_heads;
  const DkItem it = load_desc(c.items, blockIdx.x / c.n_kv_heads);
  const DkEntry e = load_desc(c.entries, it.entry);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int last_row = it.row0 + it.nrows - 1;
  const int wave_row0 = it.row0 + wave * (MB * 32);
  const bool wave_active = wave_row0 <= last_row;
  const int wave_min_limit = e.n + (min(wave_row0, last_row) >> c.gshift);
  // keys at positions above this are invisible to every row of the wavefront: those tiles are skipped
  const int wave_max_limit = wave_active ? e.n + (min(wave_row0 + MB * 32 - 1, last_row) >> c.gshift) : -1;

  bf16x8 qf[MB][8];
  int limit[MB];
  load_q<MB>(c, e, g, wave_row0, last_row, lane, qf, limit);
  // From here on Q is only ever an AGPR operand: give it its home there, once, instead of a copy per use.
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+a"(qf[mb][ks]));

  WaveState st;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    st.m[mb] = -INFINITY;
    st.l[mb] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      f32x16 z = {0};
      asm volatile("" : "+a"(z));  // born in an AGPR tuple as a whole
      st.o[db][mb] = z;
    }
  }
  const uint32_t koff = k_lane_off(lane), voff = v_lane_off(lane);

  // LDS ring of 4 stages; tile t lives in stage t % 4.  Step t needs V of tile t and K of tile t+1,
  // so before step t every wavefront waits for its own share of tile t+1, then the barrier makes the
  // whole tile visible and proves that step t-1 is finished everywhere, which frees stage (t+3) % 4
  // for the loads of tile t+3.
  KvCursor cur{c.segs, e.seg_begin, e.seg_end, it.kv_lo, it.kv_hi};
  auto issue = [&](const KvTile& t, int stage) {
    char* kl = smem + stage * TILE_STAGE_BYTES;
    char* vl = kl + TILE_KT * ROW_BYTES;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      load_rows4<false>(t.k, t.stride, t.cnt, kl, wave + 4 * b, lane);
      load_rows4<true>(t.v, t.stride, t.cnt, vl, wave + 4 * b, lane);
    }
  };
  // (cnt, pos) of the tile being computed and of the two after it; pos < 0 marks "no such tile"
  int cnt0 = 0, pos0 = -1, cnt1 = 0, pos1 = -1, cnt2 = 0, pos2 = -1;
  {
    KvTile t;
    if (cur.next(c, g, TILE_KT, t)) { issue(t, 0); cnt0 = t.cnt; pos0 = t.pos; }
    if (pos0 >= 0 && cur.next(c, g, TILE_KT, t)) { issue(t, 1); cnt1 = t.cnt; pos1 = t.pos; }
    if (pos1 >= 0 && cur.next(c, g, TILE_KT, t)) { issue(t, 2); cnt2 = t.cnt; pos2 = t.pos; }
  }
  f32x16 sa[2][MB], sb[2][MB];

  // prologue: S^T of tile 0
  if (pos2 >= 0) wait_vmcnt<16>(); else if (pos1 >= 0) wait_vmcnt<8>(); else wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  if (pos0 >= 0 && pos0 <= wave_max_limit) {
    const char* kl = smem;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 a0 = read_k_frag(kl, koff, 0, ks);
      const bf16x8 a1 = read_k_frag(kl, koff, 1, ks);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        if (ks == 0) {
          mfma_s_first(sa[0][mb], a0, qf[mb][0]);
          mfma_s_first(sa[1][mb], a1, qf[mb][0]);
        } else {
          mfma_s(sa[0][mb], a0, qf[mb][ks]);
          mfma_s(sa[1][mb], a1, qf[mb][ks]);
        }
      }
    }
    settle(sa[0][0], sa[0][1], sa[1][0], sa[1][1]);
  }

  int stage = 0;  // stage of the tile being computed
  while (pos0 >= 0) {
    // tile t+1 must have landed (tile t+2 may still be in flight)
    if (pos2 >= 0) wait_vmcnt<8>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    int cnt3 = 0, pos3 = -1;
    {
      KvTile t;
      if (pos2 >= 0 && cur.next(c, g, TILE_KT, t)) { issue(t, (stage + 3) & 3); cnt3 = t.cnt; pos3 = t.pos; }
    }
    if (pos0 <= wave_max_limit) {
      const char* vl = smem + stage * TILE_STAGE_BYTES + TILE_KT * ROW_BYTES;
      const char* kn = smem + ((stage + 1) & 3) * TILE_STAGE_BYTES;
      const bool need_mask = cnt0 < TILE_KT || pos0 + TILE_KT - 1 > wave_min_limit;
      tile_step(kn, vl, qf, sa, sb, st, limit, c.c, lane, cnt0, pos0, need_mask, koff, voff);
    }
    cnt0 = cnt1; pos0 = pos1;
    cnt1 = cnt2; pos1 = pos2;
    cnt2 = cnt3; pos2 = pos3;
    stage = (stage + 1) & 3;
  }

  if (wave_active) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) settle_acc(st.o[db][mb]);
    float ltot[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) ltot[mb] = st.l[mb] + __shfl_xor(st.l[mb], 32);
#pragma unroll
    for (int db = 0; db < 4; ++db) store_block<MB>(c, e, it, g, wave * (MB * 32), lane, db, st.o[db], ltot);
    store_ml<MB>(c, e, it, g, wave * (MB * 32), lane, st.m, ltot);
  }
}

}  // namespace mfma

hipError_t launch_attend_tile(const AttendArgs& a, const DkItem* items, int32_t n_items, hipStream_t stream) {
  using namespace mfma;
  if (n_items <= 0) return hipSuccess;
  if (a.arena.head_dim != D || a.arena.dtype != 1) return hipErrorInvalidValue;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)attend_tile_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       TILE_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const Ctx c = make_ctx(a, items);
  attend_tile_kernel<<<dim3((unsigned)n_items * a.arena.n_kv_heads), 256, TILE_LDS_BYTES, stream>>>(c);
  return hipGetLastError();
}

}  // namespace dk
