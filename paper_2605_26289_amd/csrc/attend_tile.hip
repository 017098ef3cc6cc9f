// bf16 MFMA delta-prefill attention, large-Delta ("tile") kernel for gfx950, head_dim 128.
//
// A workgroup owns 256 packed query rows of one KV head (4 wavefronts x 64 rows, row r = token r / G,
// head r % G of the group) and walks the visible keys in 64-key tiles that all four wavefronts share
// through LDS (HBM -> LDS by global_load_lds_dwordx4, one barrier per tile).
//
// Per tile and wavefront there are 64 MFMAs (32 for S^T = K Q^T, 32 for O^T += V^T P^T, all
// v_mfma_f32_32x32x16_bf16) and 64 score elements per lane for the softmax.  With one wavefront per
// SIMD the matrix pipe only stays busy if the same instruction stream feeds it while doing the
// softmax, so the key loop is a three-stage software pipeline.  Step t issues
//     S^T(t+1)             32 MFMAs, K tile t+1
//     O^T += V^T P^T(t-1)  32 MFMAs, V tile t-1 and the probabilities made in step t-1
// and, between those MFMAs, the VALU turns S^T(t) into P(t) (exp2, bf16 pack, row sums) and takes the
// row maxima of S^T(t+1) once that is complete.  Nothing inside a step depends on anything else
// computed in the same step, so the interleaving is a static schedule: a few VALU / LDS instructions
// after every MFMA.
//
// The reference maximum of a row only has to be raised when the scores outgrow it by more than
// RESCALE_SLACK; whether tile t needs that is known before step t starts (its maxima were taken in
// step t-1).  Raising it is rare after the first tile and costs nothing inside the step: the weight
// sum is rescaled on the spot, P(t) is made against the new maximum, and O -- which in step t still
// receives P(t-1), made against the old one -- is rescaled at the top of step t+1.
// There is one step body for everything.  Tiles on the causal diagonal or with a ragged end get their
// hidden scores set to -inf before the step; a tile a wavefront cannot see at all (its rows end
// earlier than those of the workgroup's other wavefronts) or that does not exist (the extra last step
// that only has P(t-1) left to apply) is simply masked completely, so its probabilities are zero.
// Step 0 applies a zero P to a zero-filled V stage.
//
// Register plan (one wavefront per SIMD, 512 registers): AGPRs hold the O^T accumulators (128) and Q
// (64, read by the MFMAs as B operand straight from AGPRs) and the K/V fragments on their way from
// LDS; VGPRs hold two S^T buffers (2 x 64, written by the MFMAs directly) and two P buffers (2 x 32).
// The step body exists twice with the buffer roles swapped, so nothing is copied between steps.
// The MFMAs are issued from inline assembly so that this placement is exactly what the compiler
// allocates; the consequence is that MFMA-result hazards are handled by hand (see settle()).
#include <hip/hip_runtime.h>

#include <mutex>
#include <utility>

#include "attend_common.hpp"
#include "kernels.hpp"

namespace dk {
namespace mfma {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr int TILE_KT = 64;
constexpr int TILE_K_RING = 3, TILE_V_RING = 5;        // stages per ring
constexpr int TILE_STAGE_BYTES = TILE_KT * ROW_BYTES;  // 16 KiB
constexpr int TILE_LDS_BYTES = (TILE_K_RING + TILE_V_RING) * TILE_STAGE_BYTES;
constexpr int MB = 2;  // 32-row blocks per wavefront

// S^T accumulators live in VGPRs, O^T accumulators and Q in AGPRs.
__device__ __forceinline__ void mfma_s_first(f32x16& s, const bf16x8& k, const bf16x8& q) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "a"(k), "a"(q));
}
__device__ __forceinline__ void mfma_s(f32x16& s, const bf16x8& k, const bf16x8& q) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "a"(k), "a"(q));
}
__device__ __forceinline__ void mfma_o(f32x16& o, const bf16x8& v, const u32x4& p) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o) : "a"(v), "v"(p));
}

// The compiler does not see that these registers come out of the matrix pipeline, so it would not
// insert the wait states a plain VALU read of a fresh MFMA result needs.  Every place where such a
// read can follow an MFMA closely passes the registers through this first.
__device__ __forceinline__ void settle(f32x16& a, f32x16& b, f32x16& c, f32x16& d) {
  asm volatile("s_nop 15\n\ts_nop 7" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}
__device__ __forceinline__ void settle_acc(f32x16& a) { asm volatile("s_nop 15\n\ts_nop 7" : "+a"(a)); }

__device__ __forceinline__ float max3(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}
// Keeps a value's computation where the source has it: ordinary arithmetic whose only consumers are
// in a later step would otherwise be sunk out of the MFMA schedule it is meant to fill.
// (Input-only on purpose: an asm that redefined the register would make the hazard recogniser pad its
// next use with a wait state.)
template <typename T>
__device__ __forceinline__ void pin(const T& x) {
  asm volatile("" : : "v"(x));
}
// max over the two half-waves: lane l and lane l ^ 32 both get max(x[l], x[l ^ 32])
__device__ __forceinline__ float max_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return max3(__uint_as_float(r[0]), __uint_as_float(r[1]), __uint_as_float(r[1]));
}
// The reference maximum of a row only moves when its maximum grew by more than this (log2 units):
// after the first tiles the rescale of O is rare, and the weights stay below 2^8.
constexpr float RESCALE_SLACK = 8.f;

#ifdef DK_PROF  // timing build: cycles per loop section, summed over wavefronts
__device__ unsigned long long g_prof[8];
#define DK_PROF_T(x) const long long x = __builtin_readcyclecounter()
#define DK_PROF_ADD(i, v) pacc[i] += (v)
#else
#define DK_PROF_T(x)
#define DK_PROF_ADD(i, v)
#endif

#ifdef DK_TRACE  // timeline build: wall-clock stamps (100 MHz) of wavefront 0 per workgroup and item
__device__ unsigned long long g_trace[256][16][8];
#define DK_TR(seq, ph)                                                                                  \
  do {                                                                                                  \
    if (threadIdx.x == 0 && (seq) < 16 && blockIdx.x < 256) g_trace[blockIdx.x][(seq)][(ph)] = wall_clock64(); \
  } while (0)
#else
#define DK_TR(seq, ph)
#endif

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

// Row maxima (unscaled) of one S^T tile.
__device__ __forceinline__ void row_max(const f32x16 (&s)[2][MB], float (&mx)[MB]) {
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    float v = max3(s[0][mb][0], s[1][mb][0], s[1][mb][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) v = max3(v, s[0][mb][r], s[1][mb][r]);
    mx[mb] = max_halves(v);
  }
}

// O *= alpha, row by row.  Whole-register arithmetic only: element-wise inserts into the accumulator
// tuples make the compiler shuttle all of O between the two register files on every trip of the key loop.
// settle_acc() pads both the read after the last MFMA and the next MFMA after the write.
__device__ __forceinline__ void rescale_o(WaveState& st, const float (&alpha)[MB]) {
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      settle_acc(st.o[db][mb]);
      f32x16 t = st.o[db][mb];
      t = t * alpha[mb];
      st.o[db][mb] = t;
      settle_acc(st.o[db][mb]);
    }
}

// HBM -> LDS loads of one step: the wavefront's share (4 x 1 KiB each) of one K tile and one V tile.
// kvo/vvo are the per-lane byte offsets inside the tile (row * stride + swizzled chunk), kept across
// steps because they only change with the tile's row count or stride.
struct TileLoads {
  uint32_t lds_k, lds_v;  // LDS byte address of the wavefront's next 1 KiB block in the target stages
  uint32_t kvo[4], vvo[4];
};

// One wavefront moves 1 KiB HBM -> LDS, lane l landing at lds_addr + 16 l.  Issued from inline assembly
// on purpose: the compiler then keeps no account of it and inserts no vmcnt(0) of its own in front of
// later LDS reads; completion is awaited explicitly with wait_vmcnt<N>().
// The wait state that must separate the write of M0 from the load is filled with the address arithmetic
// for the wavefront's next block (4 KiB further on in the stage), so a block costs two issue slots.
__device__ __forceinline__ void dma16_advance(const char* gbase, uint32_t voff, uint32_t& lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_add_i32 %0, %0, 0x1000\n\t"
      "global_load_lds_dwordx4 %1, %2"
      : "+s"(lds_addr)
      : "v"(voff), "s"(gbase)
      : "memory", "m0", "scc");
}
// The tile kernel's walk over an item's key positions [p, hi): like KvCursor, but the current tile lives in
// the cursor itself (k, v, stride, cnt, pos: no copy per step) and the usual step -- another full tile of the
// same segment -- is a compare, two pointer additions and two counter updates.
struct TileCursor {
  const DkSeg* segs;
  int32_t si, se, p, hi;  // p: first position after the current tile
  int32_t seg_end = 0;    // first position past the current segment (0: no segment loaded yet)
  int32_t full_end = 0;   // min(seg_end, hi): a full tile fits while p + TILE_KT <= full_end
  const char* k = nullptr;  // current tile
  const char* v = nullptr;
  uint32_t stride = 0;  // bytes between consecutive rows
  uint32_t adv = 0;     // bytes from the current tile to the next one of the same segment
  int32_t cnt = 0;      // valid rows of the current tile
  int32_t pos = 0;      // logical position of its row 0

  // Moves on to the next tile; false (and the current tile stays) when the range is exhausted.
  __device__ __forceinline__ bool next(const Ctx& c, int g) {
    if (p + TILE_KT <= full_end) {  // cnt stays TILE_KT, adv stays TILE_KT * stride
      k += adv;
      v += adv;
      pos = p;
      p += TILE_KT;
      return true;
    }
    if (p >= hi) return false;
    if (p >= seg_end) {
      DkSeg s = load_desc(segs, si);
      while (s.pos + s.len <= p && si + 1 < se) s = load_desc(segs, ++si);
      const int32_t off = p - s.pos;
      seg_end = s.pos + s.len;
      full_end = min(seg_end, hi);
      if (s.src == 0) {
        const int64_t byte = ((int64_t)g * c.arena_cells + s.start + off) * ROW_BYTES;
        k = c.k_arena + byte;
        v = c.v_arena + byte;
        stride = ROW_BYTES;
      } else {
        const int64_t byte = ((s.start + off) * c.n_kv_heads + g) * (int64_t)ROW_BYTES;
        k = c.k_new + byte;
        v = c.v_new + byte;
        stride = (uint32_t)c.n_kv_heads * ROW_BYTES;
      }
    } else {
      k += adv;
      v += adv;
    }
    cnt = min(TILE_KT, full_end - p);
    pos = p;
    p += cnt;
    adv = (uint32_t)cnt * stride;
    return true;
  }
};

template <int I>
__device__ __forceinline__ void issue_one(TileLoads& ld, const TileCursor& cur) {
  if constexpr (I < 4) dma16_advance(cur.k, ld.kvo[I], ld.lds_k);
  else dma16_advance(cur.v, ld.vvo[I - 4], ld.lds_v);
}
// Per-lane offsets of the wavefront's four blocks of a tile with cnt rows: block b is rows
// 16 b + 4 wave + lane / 16, lane l fetching the chunk that the swizzle assigns to slot l % 16.
// Rows past the end of a ragged tile re-read the last valid row; their scores are masked.
template <bool IS_V>
__device__ __forceinline__ void lane_offsets(uint32_t (&vo)[4], int wave, int lane, int cnt, uint32_t stride) {
  const int row0 = wave * 4 + (lane >> 4);
  const int slot = lane & 15;
  const int chunk = IS_V ? (slot ^ ((row0 & 3) << 2)) : (slot ^ (row0 & 15));
#pragma unroll
  for (int b = 0; b < 4; ++b) vo[b] = (uint32_t)min(row0 + 16 * b, cnt - 1) * stride + chunk * 16;
}

// ---- pipelined step ----------------------------------------------------------------------------------
//   MFMA  0..31  S^T(next): depth step i/4, key block (i/2)%2, row block i%2
//   MFMA 32..63  PV(prev):  key step j = (i-32)/8, depth block ((i-32)/2)%4, row block i%2
// VALU work of the current tile: slot i exponentiates element i and scales element i+1; every second
// slot packs the pair finished one slot earlier; the row sum takes each weight one slot after its exp2.
// LDS reads: K fragments two depth steps (eight slots) ahead; V fragments two (j, db) pairs at a time,
// eight slots ahead of their first use.  Each group is awaited once, at its first use.
struct FastStep {
  const char* k_lds;  // K tile t+1
  const char* v_lds;  // V tile t-1
  const bf16x8 (&qf)[MB][8];
  f32x16 (&sc)[2][MB];
  f32x16 (&sn)[2][MB];
  const u32x4 (&pp)[MB][4];
  u32x4 (&pc)[MB][4];
  WaveState& st;
  TileLoads& ld;
  const TileCursor& cur;
  const float (&ms)[MB];
  float c;
  uint32_t koff, voff;
  float mxn[MB];
  float xe[2];      // scaled scores waiting for their exp2
  float pe[2][2];   // [pair parity][element]
  bf16x8 kf[3][2];  // [depth step % 3][key block]
  bf16x8 vf[6];     // ring over the (j, db) pairs

  // Softmax element E (0..63) of the current tile, in the order PV will consume them: pair E/2 is one
  // bf16 register of P.  The four instructions of an element's chain (multiply-add, exp2, pack, row sum)
  // run in different slots, each at least one slot after the one that feeds it, so none of them waits
  // on its predecessor's result.
  template <int E>
  __device__ __forceinline__ void scale() {
    constexpr int Q = E >> 1, HALF = E & 1;
    constexpr int grp = Q >> 2, w = Q & 3;
    constexpr int mb = grp & 1, j = grp >> 1;
    constexpr int kb = j >> 1, r = 8 * (j & 1) + 2 * w + HALF;
    xe[E & 1] = __builtin_fmaf(sc[kb][mb][r], c, -ms[mb]);
    pin(xe[E & 1]);
  }
  template <int E>
  __device__ __forceinline__ void expo() {
    float p = __builtin_amdgcn_exp2f(xe[E & 1]);
    pin(p);
    pe[(E >> 1) & 1][E & 1] = p;
  }
  // Row sums are plain fp32 adds of the unrounded weights, one slot after the exp2.  (Summing the rounded
  // pair with a v_dot2 would be half the instructions, but the dot instructions run on the matrix pipe:
  // measured, each one stalls until the MFMA in flight has drained.)
  template <int E>
  __device__ __forceinline__ void rowsum() {
    constexpr int mb = (E >> 3) & 1;
    st.l[mb] += pe[(E >> 1) & 1][E & 1];
    pin(st.l[mb]);
  }
  template <int Q>
  __device__ __forceinline__ void pack() {
    constexpr int grp = Q >> 2, w = Q & 3;
    constexpr int mb = grp & 1, j = grp >> 1;
    bf16x2 pw;
    pw[0] = (__bf16)pe[Q & 1][0];
    pw[1] = (__bf16)pe[Q & 1][1];
    const uint32_t word = __builtin_bit_cast(uint32_t, pw);
    pin(word);
    pc[mb][j][w] = word;
  }
  // row maxima of the next tile: op Z of 32 chained max3 (Z % 2 = row block), then the half-wave exchange
  template <int Z>
  __device__ __forceinline__ void maxop() {
    if constexpr (Z < 32) {
      constexpr int mb = Z & 1, k = Z >> 1;
      if constexpr (k == 0) mxn[mb] = max3(sn[0][mb][0], sn[1][mb][0], sn[1][mb][0]);
      else mxn[mb] = max3(mxn[mb], sn[0][mb][k], sn[1][mb][k]);
    } else {
      mxn[Z - 32] = max_halves(mxn[Z - 32]);
    }
  }
  static constexpr int MAX_FIRST = 36;  // first slot with row-maximum work (S^T(next) is complete and settled)
  static constexpr int zslot(int z) { return MAX_FIRST + z * (64 - MAX_FIRST) / 34; }

  template <int I, int... Zs>
  __device__ __forceinline__ void run_max(std::integer_sequence<int, Zs...>) {
    ((zslot(Zs) == I ? maxop<Zs>() : (void)0), ...);
  }
  template <int PAIR>
  __device__ __forceinline__ void read_v_pair() {
    vf[PAIR % 6] = read_v_frag(v_lds, voff, PAIR >> 2, PAIR & 3);
  }

  template <int I>
  __device__ __forceinline__ void slot() {
    if constexpr (I < 32) {
      constexpr int ks = I >> 2, kb = (I >> 1) & 1, mb = I & 1;
      if constexpr ((I & 3) == 0) {
        if constexpr (ks + 2 < 8) {
          kf[(ks + 2) % 3][0] = read_k_frag(k_lds, koff, 0, ks + 2);
          kf[(ks + 2) % 3][1] = read_k_frag(k_lds, koff, 1, ks + 2);
        }
        // one wait for both key blocks of this depth step
        asm volatile("" : : "a"(kf[ks % 3][0]), "a"(kf[ks % 3][1]));
      }
      if constexpr (ks == 0) mfma_s_first(sn[kb][mb], kf[0][kb], qf[mb][0]);
      else mfma_s(sn[kb][mb], kf[ks % 3][kb], qf[mb][ks]);
      if constexpr (I == 24) {
        read_v_pair<0>();
        read_v_pair<1>();
      }
      if constexpr (I == 28) {
        read_v_pair<2>();
        read_v_pair<3>();
      }
    } else {
      constexpr int pair = (I - 32) >> 1, mb = I & 1;  // pair = j * 4 + db
      constexpr int j = pair >> 2, db = pair & 3;
      if constexpr (((I - 32) & 3) == 0) {
        if constexpr (pair + 4 < 16) {
          read_v_pair<pair + 4>();
          read_v_pair<pair + 5>();
        }
        asm volatile("" : : "a"(vf[pair % 6]), "a"(vf[(pair + 1) % 6]));
      }
      mfma_o(st.o[db][mb], vf[pair % 6], pp[mb][j]);
    }
    // softmax of the current tile
    expo<I>();
    if constexpr (I + 1 < 64) scale<I + 1>();
    if constexpr (I >= 1) rowsum<I - 1>();
    if constexpr ((I & 1) == 0 && I >= 2) pack<I / 2 - 1>();
    // HBM -> LDS loads of later tiles
    if constexpr ((I & 1) == 1 && I < 16) issue_one<(I - 1) / 2>(ld, cur);
    // row maxima of the next tile
    if constexpr (I >= MAX_FIRST) run_max<I>(std::make_integer_sequence<int, 34>{});
    __builtin_amdgcn_sched_barrier(0);
  }

  template <int... Is>
  __device__ __forceinline__ void run(std::integer_sequence<int, Is...>) {
    (slot<Is>(), ...);
  }
  template <int BASE, int... Is>
  __device__ __forceinline__ void run_from(std::integer_sequence<int, Is...>) {
    (slot<BASE + Is>(), ...);
  }
};

// S^T of one tile, nothing overlapped.
__device__ __forceinline__ void plain_s(const char* k_lds, const bf16x8 (&qf)[MB][8], f32x16 (&s)[2][MB],
                                        uint32_t koff) {
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const bf16x8 a0 = read_k_frag(k_lds, koff, 0, ks);
    const bf16x8 a1 = read_k_frag(k_lds, koff, 1, ks);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      if (ks == 0) {
        mfma_s_first(s[0][mb], a0, qf[mb][0]);
        mfma_s_first(s[1][mb], a1, qf[mb][0]);
      } else {
        mfma_s(s[0][mb], a0, qf[mb][ks]);
        mfma_s(s[1][mb], a1, qf[mb][ks]);
      }
    }
  }
  settle(s[0][0], s[0][1], s[1][0], s[1][1]);
}

// grid = n_chains * n_kv_heads workgroups, at most one per compute unit: workgroup w serves KV head
// w % n_kv_heads (with 8 KV heads that is also the XCD it lands on, so all row tiles of a head share one
// L2) and walks chain w / n_kv_heads of work items: links[chain], links[n_chains + item], ... until a
// link is negative.  The chains are the same for every KV head; the planner balanced them.
// Between two items of a chain the loads of the next item (descriptors, Q, its first two K/V tiles) are
// requested before the output of the finished one is stored, so they overlap with the store phase.
// INLINE: the descriptors arrive inside the kernel arguments (first argument) and the descriptor pointers are
// byte offsets into them; otherwise they point into the uploaded workspace.
template <bool INLINE>
__global__ __launch_bounds__(256, 1) void attend_tile_kernel(BlobArg<INLINE> blob, Ctx c, const int32_t* links,
                                                             int n_chains) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  (void)blob;
  c.entries = resolve_desc<INLINE>(c.entries);
  c.segs = resolve_desc<INLINE>(c.segs);
  c.items = resolve_desc<INLINE>(c.items);
  links = resolve_desc<INLINE>(links);
  const int g = blockIdx.x % c.n_kv_heads;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t koff = k_lane_off(lane), voff = v_lane_off(lane);

  // Two LDS rings of 16 KiB stages: K tile u lives in stage u % 3 of the K ring, V tile u in stage
  // u % 5 of the V ring.  Step t reads K(t+1) and V(t-1) and requests tile t+3 (K and V), i.e. every
  // tile is requested two steps before its first use.  The barrier at the top of step t proves step
  // t-1 is finished everywhere, which is what frees the stages of K(t) and V(t-2) for those loads.
  // Past the end of the key range the last tile is simply loaded again (into stages nobody reads any
  // more), so that every step leaves exactly eight loads per wavefront in flight and one wait count
  // fits all steps.
  char* const k_ring = smem;
  char* const v_ring = smem + TILE_K_RING * TILE_STAGE_BYTES;
  const uint32_t k_ring_lds = (uint32_t)(uintptr_t)(lds_void_ptr)k_ring + wave * 1024;
  const uint32_t v_ring_lds = (uint32_t)(uintptr_t)(lds_void_ptr)v_ring + wave * 1024;

  // ---- state of the item being worked on (set by begin_item) -------------------------------------
  DkItem it;
  DkEntry e;
  int last_row = 0, wave_min_limit = 0, wave_max_limit = -1;
  bool wave_active = false;
  bf16x8 qf[MB][8];
  int limit[MB];
  TileCursor cur{c.segs, 0, 0, 0, 0};  // its current tile is the next one to load
  TileLoads ld;
  int ld_cnt = -1;
  uint32_t ld_stride = 0;
  // (cnt, pos) of tiles t .. t+2 of the step about to run; cnt 0 = no such tile
  int cnt0 = 0, pos0 = 0, cnt1 = 0, pos1 = 0, cnt2 = 0, pos2 = 0;

  auto offsets_stale = [&]() { return cur.cnt != ld_cnt || cur.stride != ld_stride; };
  auto refresh_offsets = [&]() {
    ld_cnt = cur.cnt;
    ld_stride = cur.stride;
    lane_offsets<false>(ld.kvo, wave, lane, ld_cnt, ld_stride);
    lane_offsets<true>(ld.vvo, wave, lane, ld_cnt, ld_stride);
  };
  auto aim = [&](int k_stage, int v_stage) {
    ld.lds_k = k_ring_lds + k_stage * TILE_STAGE_BYTES;
    ld.lds_v = v_ring_lds + v_stage * TILE_STAGE_BYTES;
  };
  auto issue_all = [&]() {
    issue_one<0>(ld, cur);
    issue_one<1>(ld, cur);
    issue_one<2>(ld, cur);
    issue_one<3>(ld, cur);
    issue_one<4>(ld, cur);
    issue_one<5>(ld, cur);
    issue_one<6>(ld, cur);
    issue_one<7>(ld, cur);
  };

  // Requests everything an item needs before its first step: Q (into registers), its first two K/V tiles
  // (stages 0 and 1 of both rings) and a zero-filled "V(-1)" (stage 4 of the V ring: step 0 multiplies a
  // zero P into it, so no stale NaN pattern may sit there).  Nothing is waited for.  Every stage of the
  // rings must be free: no wavefront of the workgroup may still read or load into them.
  auto begin_item = [&](const DkItem& item, const DkEntry& entry) __attribute__((always_inline)) {
    it = item;
    e = entry;
    last_row = it.row0 + it.nrows - 1;
    const int wave_row0 = it.row0 + wave * (MB * 32);
    wave_active = wave_row0 <= last_row;
    wave_min_limit = e.n + (min(wave_row0, last_row) >> c.gshift);
    // keys at positions above this are invisible to every row of the wavefront: those tiles are skipped
    wave_max_limit = wave_active ? e.n + (min(wave_row0 + MB * 32 - 1, last_row) >> c.gshift) : -1;
    load_q<MB>(c, e, g, wave_row0, last_row, lane, qf, limit);
    cur = TileCursor{c.segs, e.seg_begin, e.seg_end, it.kv_lo, it.kv_hi};
    cnt0 = pos0 = cnt2 = pos2 = 0;
    (void)cur.next(c, g);  // the planner never produces an empty key range
    cnt1 = cur.cnt;  // becomes tile 0 when step -1 hands over to step 0
    pos1 = cur.pos;
    refresh_offsets();
    aim(0, 0);
    issue_all();
    if (cur.next(c, g)) {  // when the range ends the old tile stays current
      cnt2 = cur.cnt;
      pos2 = cur.pos;
    }
    if (offsets_stale()) refresh_offsets();
    aim(1, 1);
    issue_all();
    u32x4* z = (u32x4*)(v_ring + 4 * TILE_STAGE_BYTES);
#pragma unroll
    for (int i = 0; i < TILE_STAGE_BYTES / (256 * 16); ++i) z[i * 256 + threadIdx.x] = u32x4{0, 0, 0, 0};
  };

  int trace_seq = 0;
  (void)trace_seq;
  DK_TR(0, 7);
  int item_idx = load_desc(links, blockIdx.x / c.n_kv_heads);
  {
    const DkItem first = load_desc(c.items, item_idx);
    begin_item(first, load_desc(c.entries, first.entry));
  }
  // small append-and-attend calls: this workgroup's share of the new rows goes into the arena now, under the
  // latency of the first item's requests
  scatter_new_rows<INLINE>(c);

  while (true) {
    // the next item of the chain: its descriptors arrive while this one is being computed
    const int next_idx = load_desc(links, n_chains + item_idx);
    DkItem next_item = it;
    DkEntry next_entry = e;
    if (next_idx >= 0) {
      next_item = load_desc(c.items, next_idx);
      next_entry = load_desc(c.entries, next_item.entry);
    }

    DK_TR(trace_seq, 0);
    wait_q<MB>(qf);
    DK_TR(trace_seq, 1);
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

    f32x16 sa[2][MB], sb[2][MB];
    u32x4 pa[MB][4], pb[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int j = 0; j < 4; ++j) pb[mb][j] = u32x4{0, 0, 0, 0};

    bool mx_valid = false, pending = false;
    float mx[MB] = {0.f, 0.f}, alpha[MB] = {1.f, 1.f};
    float ms[MB] = {0.f, 0.f};  // the reference maxima as subtracted from the scores: m, or 0 while m = -inf
    float gval = 0.f;           // how far the tile's scores outgrow the reference maxima (log2 units)

    // step -1: S^T(0); requests tile 2
    int cnt3 = 0, pos3 = 0;
    auto fetch = [&]() {
      cnt3 = 0;
      if (cur.next(c, g)) {
        cnt3 = cur.cnt;
        pos3 = cur.pos;
      }
    };
    fetch();
    wait_vmcnt<8>();
    __builtin_amdgcn_s_barrier();
    if (offsets_stale()) refresh_offsets();
    aim(2, 2);
    issue_all();
    if (wave_active) plain_s(k_ring, qf, sa, koff);
    cnt0 = cnt1; pos0 = pos1;
    cnt1 = cnt2; pos1 = pos2;
    cnt2 = cnt3; pos2 = pos3;
    fetch();

    DK_TR(trace_seq, 2);
    // byte offsets of the stages step t uses: K(t+1) read, K(t+3) written; V(t-1) read, V(t+3) written
    int k_rd = 1 * TILE_STAGE_BYTES, k_wr = 0, v_rd = 4 * TILE_STAGE_BYTES, v_wr = 3 * TILE_STAGE_BYTES;
#ifdef DK_PROF
    long long pacc[6] = {0, 0, 0, 0, 0, 0};
    const long long pstart = __builtin_readcyclecounter();
    const long long wstart = wall_clock64();
#endif

    // on to step t+1
    auto advance = [&]() __attribute__((always_inline)) {
      cnt0 = cnt1; pos0 = pos1;
      cnt1 = cnt2; pos1 = pos2;
      cnt2 = cnt3; pos2 = pos3;
      fetch();
      k_rd = k_rd == (TILE_K_RING - 1) * TILE_STAGE_BYTES ? 0 : k_rd + TILE_STAGE_BYTES;
      k_wr = k_wr == (TILE_K_RING - 1) * TILE_STAGE_BYTES ? 0 : k_wr + TILE_STAGE_BYTES;
      v_rd = v_rd == (TILE_V_RING - 1) * TILE_STAGE_BYTES ? 0 : v_rd + TILE_STAGE_BYTES;
      v_wr = v_wr == (TILE_V_RING - 1) * TILE_STAGE_BYTES ? 0 : v_wr + TILE_STAGE_BYTES;
    };
    auto step = [&](f32x16(&sc)[2][MB], f32x16(&sn)[2][MB], u32x4(&pp)[MB][4], u32x4(&pc)[MB][4])
                    __attribute__((always_inline)) {
      wait_vmcnt<8>();
      __builtin_amdgcn_s_barrier();
      DK_PROF_T(t1);
      const char* k_lds = k_ring + k_rd;
      const char* v_lds = v_ring + v_rd;
      ld.lds_k = k_ring_lds + k_wr;
      ld.lds_v = v_ring_lds + v_wr;
      if (!wave_active) {
        // A wavefront whose rows lie past the end of a ragged row tile only does its share of the loads and
        // keeps the barriers: no arithmetic, so it draws no matrix-pipe power either.
        if (offsets_stale()) refresh_offsets();
        issue_all();
        advance();
        return;
      }
      // a tile that does not exist or lies beyond the wavefront's rows counts as having no valid key
      const int cnt_eff = pos0 <= wave_max_limit ? cnt0 : 0;
      const bool need_mask = cnt_eff < TILE_KT || pos0 + TILE_KT - 1 > wave_min_limit;
      if (pending || need_mask || !mx_valid || offsets_stale()) {  // rare, all of it
        if (offsets_stale()) refresh_offsets();
        if (pending) {  // O still carries the reference maxima of two steps ago
          rescale_o(st, alpha);
          pending = false;
        }
        if (need_mask) mask_tile(sc, limit, lane, cnt_eff, pos0);
        if (need_mask || !mx_valid) {
          row_max(sc, mx);
          gval = fmaxf(__builtin_fmaf(mx[0], c.c, -st.m[0]), __builtin_fmaf(mx[1], c.c, -st.m[1]));
        }
      }
      if (__builtin_amdgcn_ballot_w64(gval > RESCALE_SLACK) != 0) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const float mn = fmaxf(st.m[mb], mx[mb] * c.c);
          const float mz = (mn == -INFINITY) ? 0.f : mn;
          alpha[mb] = __builtin_amdgcn_exp2f(st.m[mb] - mz);  // 1 for rows whose maximum did not move
          st.m[mb] = mn;
          ms[mb] = mz;
          st.l[mb] *= alpha[mb];
        }
        pending = true;
      }
      DK_PROF_T(t2);
      {
        FastStep f{k_lds, v_lds, qf, sc, sn, pp, pc, st, ld, cur, ms, c.c, koff, voff};
        f.kf[0][0] = read_k_frag(k_lds, koff, 0, 0);
        f.kf[0][1] = read_k_frag(k_lds, koff, 1, 0);
        f.kf[1][0] = read_k_frag(k_lds, koff, 0, 1);
        f.kf[1][1] = read_k_frag(k_lds, koff, 1, 1);
        __builtin_amdgcn_sched_barrier(0);
        f.scale<0>();
#ifdef DK_PROF
        f.run(std::make_integer_sequence<int, 32>{});
        DK_PROF_T(tm);
        DK_PROF_ADD(1, tm - t2);
        f.run_from<32>(std::make_integer_sequence<int, 32>{});
#else
        f.run(std::make_integer_sequence<int, 64>{});
#endif
        f.rowsum<63>();
        f.pack<31>();
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) mx[mb] = f.mxn[mb];
        // -inf - -inf for rows that have seen no key yet: NaN compares false, which is right (nothing to raise)
        gval = fmaxf(__builtin_fmaf(mx[0], c.c, -st.m[0]), __builtin_fmaf(mx[1], c.c, -st.m[1]));
        mx_valid = true;
      }
      DK_PROF_T(t3);
      DK_PROF_ADD(2, t3 - t1);
      DK_PROF_ADD(3, 1);
      advance();
    };

    // steps 0 .. T for T tiles: the last one only applies P(T-1)
    while (true) {
      bool last = cnt0 == 0;
      step(sa, sb, pb, pa);
      if (last) break;
      last = cnt0 == 0;
      step(sb, sa, pa, pb);
      if (last) break;
    }
    if (pending) rescale_o(st, alpha);
    wait_vmcnt<0>();
    DK_TR(trace_seq, 3);

#ifdef DK_PROF
    if (lane == 0) {
      atomicAdd(&g_prof[0], (unsigned long long)(__builtin_readcyclecounter() - pstart));
      atomicAdd(&g_prof[2], (unsigned long long)pacc[1]);
      atomicAdd(&g_prof[3], (unsigned long long)pacc[2]);
      atomicAdd(&g_prof[4], (unsigned long long)pacc[3]);
      atomicAdd(&g_prof[6], (unsigned long long)(wall_clock64() - wstart));
    }
#endif
    // what the store below needs of the finished item
    const DkItem done_item = it;
    const DkEntry done_entry = e;
    const bool done_active = wave_active;
    // Every wavefront has left the last step: the rings are free.  The next item's first loads are requested
    // now and travel while this item's output is being stored; the store is staged through the part of the V
    // ring those loads do not touch (stages 2 and 3, 8 KiB per wavefront).
    __builtin_amdgcn_s_barrier();
    if (next_idx >= 0) begin_item(next_item, next_entry);
    DK_TR(trace_seq, 4);
    if (done_active) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) settle_acc(st.o[db][mb]);
      float ltot[MB];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) ltot[mb] = st.l[mb] + __shfl_xor(st.l[mb], 32);
      // (the lane number is laundered so that the store phase's per-lane offsets are computed here, each time,
      // instead of being hoisted out of the item loop, where they would sit in registers the key loop needs)
      int store_lane = lane;
      asm volatile("" : "+v"(store_lane));
      store_rows_staged<MB>(c, done_entry, done_item, g, wave * (MB * 32), store_lane,
                            v_ring + 2 * TILE_STAGE_BYTES + wave * 8192, st.o, ltot);
      store_ml<MB>(c, done_entry, done_item, g, wave * (MB * 32), store_lane, st.m, ltot);
    }
    DK_TR(trace_seq, 5);
#ifdef DK_TRACE
    if (threadIdx.x == 0 && trace_seq < 16 && blockIdx.x < 256)
      g_trace[blockIdx.x][trace_seq][6] = (unsigned long long)((done_item.kv_hi - done_item.kv_lo + 63) / 64);
    ++trace_seq;
#endif
    if (next_idx < 0) break;
    item_idx = next_idx;
  }
}

}  // namespace mfma

hipError_t launch_attend_tile(const AttendArgs& a, const DkItem* items, const int32_t* links, int32_t n_chains,
                              hipStream_t stream) {
  using namespace mfma;
  if (n_chains <= 0) return hipSuccess;
  if (a.arena.head_dim != D || a.arena.dtype != 1) return hipErrorInvalidValue;
  // once per process, whatever thread or pool gets here first
  static std::once_flag attr_once;
  static hipError_t attr_status = hipSuccess;
  std::call_once(attr_once, [] {
    attr_status = hipFuncSetAttribute((const void*)attend_tile_kernel<false>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, TILE_LDS_BYTES);
    if (attr_status == hipSuccess)
      attr_status = hipFuncSetAttribute((const void*)attend_tile_kernel<true>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, TILE_LDS_BYTES);
  });
  if (attr_status != hipSuccess) return attr_status;
  const Ctx c = make_ctx(a, items);
  const dim3 grid((unsigned)n_chains * a.arena.n_kv_heads);
  if (a.inline_blob) {
    BlobArg<true> blob{*a.inline_blob};
    attend_tile_kernel<true><<<grid, 256, TILE_LDS_BYTES, stream>>>(blob, c, links, n_chains);
  } else {
    attend_tile_kernel<false><<<grid, 256, TILE_LDS_BYTES, stream>>>(BlobArg<false>{0}, c, links, n_chains);
  }
  return hipGetLastError();
}

}  // namespace dk
