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

#include "kernels.hpp"

namespace dk {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(3))) bf16x4* lds_bf16x4_ptr;
typedef __attribute__((address_space(1))) const void* glb_void_ptr;

constexpr int D = 128;
constexpr int ROW_BYTES = 256;
constexpr int PS = D + 2;  // floats per partial row: D sums, running max (log2 units), weight sum

// Descriptors are read through the constant address space so that uniform reads become scalar loads
// (they must not take part in the vector-memory counter that tracks the K/V tiles in flight).
template <typename T>
__device__ __forceinline__ T load_desc(const T* base, int idx) {
  static_assert(sizeof(T) % 4 == 0, "descriptor structs are made of 32-bit words");
  typedef const __attribute__((address_space(4))) uint32_t* const_u32_ptr;
  const_u32_ptr p = (const_u32_ptr)((uintptr_t)base + (size_t)idx * sizeof(T));
  T out;
  uint32_t* o = (uint32_t*)&out;
#pragma unroll
  for (unsigned i = 0; i < sizeof(T) / 4; ++i) o[i] = p[i];
  return out;
}

struct Ctx {
  const DkEntry* entries;
  const DkSeg* segs;
  const DkItem* items;
  const __bf16* __restrict__ q;
  const char* __restrict__ k_arena;
  const char* __restrict__ v_arena;
  const char* __restrict__ k_new;
  const char* __restrict__ v_new;
  __bf16* __restrict__ out;
  float* __restrict__ lse;
  float* __restrict__ parts;
  float c;  // softmax scale * log2(e): scores are handled in log2 units
  int32_t n_q_heads, n_kv_heads, gshift;
  int64_t arena_cells;
};

// A run of at most KT consecutive K/V rows, all inside one segment.
struct KvTile {
  const char* k;
  const char* v;
  uint32_t stride;  // bytes between consecutive rows
  int32_t cnt;      // valid rows (>= 1)
  int32_t pos;      // logical position of row 0
};

// Walks the logical key positions [p, hi) of an entry, segment by segment.
struct KvCursor {
  const DkSeg* segs;
  int32_t si, se, p, hi;

  __device__ bool next(const Ctx& c, int g, int kt, KvTile& t) {
    if (p >= hi) return false;
    DkSeg s = load_desc(segs, si);
    while (s.pos + s.len <= p && si + 1 < se) s = load_desc(segs, ++si);
    const int32_t off = p - s.pos;
    t.cnt = min(kt, min(s.pos + s.len, hi) - p);
    if (s.src == 0) {
      const int64_t byte = ((int64_t)g * c.arena_cells + s.start + off) * ROW_BYTES;
      t.k = c.k_arena + byte;
      t.v = c.v_arena + byte;
      t.stride = ROW_BYTES;
    } else {
      const int64_t byte = ((s.start + off) * c.n_kv_heads + g) * (int64_t)ROW_BYTES;
      t.k = c.k_new + byte;
      t.v = c.v_new + byte;
      t.stride = (uint32_t)c.n_kv_heads * ROW_BYTES;
    }
    t.pos = p;
    p += t.cnt;
    return true;
  }
};

// One wavefront moves 4 rows (1 KiB) HBM -> LDS: lane l lands at lds + 16 l, i.e. row l / 16, chunk
// slot l % 16, and fetches the chunk that the swizzle assigns to that slot.  Rows past the end of a
// ragged tile re-read the last valid row; their scores are masked.
// The load is issued from inline assembly on purpose: the compiler then keeps no account of it and
// inserts no vmcnt(0) of its own in front of later LDS reads, so a tile can stay in flight while
// the previous one is being consumed.  Completion is awaited explicitly with wait_vmcnt<N>().
template <bool IS_V>
__device__ __forceinline__ void load_rows4(const char* gbase, uint32_t stride, int cnt, char* lds_region, int blk,
                                           int lane) {
  const int row = blk * 4 + (lane >> 4);
  const int slot = lane & 15;
  const int chunk = IS_V ? (slot ^ ((row & 3) << 2)) : (slot ^ (row & 15));
  const uint32_t voff = (uint32_t)min(row, cnt - 1) * stride + chunk * 16;
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_void_ptr)(lds_region + blk * 1024);
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_addr), "v"(voff), "s"(gbase)
      : "memory", "m0");
}

// A operand of S^T = K Q^T for key block kb and depth step ks: lane (row l%32, half h = l/32) holds
// K[kb*32 + l%32][ks*16 + 8h .. +7], which the swizzle keeps in chunk (2ks + h) ^ (row & 15) of its row.
// Because 2ks has bit 0 clear, that chunk is (2ks) ^ (h ^ (row & 15)): the per-lane part of the address
// is computed once (k_lane_off) and each depth step only XORs in ks << 5.
__device__ __forceinline__ uint32_t k_lane_off(int lane) {
  const int r = lane & 31;
  return (uint32_t)(r * ROW_BYTES + (((lane >> 5) ^ (r & 15)) << 4));
}
__device__ __forceinline__ bf16x8 read_k_frag(const char* k_lds, uint32_t lane_off, int kb, int ks) {
  return *(const bf16x8*)(k_lds + (lane_off ^ (uint32_t)(ks << 5)) + kb * (32 * ROW_BYTES));
}

// A operand of O^T = V^T P^T for key step j (16 keys) and depth block db: lane (column l%32, half
// h = l/32) holds V[16j + 8u + 4h + e][db*32 + l%32] for u = 0,1 and e = 0..3 -- the same key order
// in which the S^T accumulators hand over P.  Two transposing 64-bit LDS reads: within 16 lanes, lane i
// supplies the address of row i/4, 4-column piece i%4 and receives column i of the four rows.
// The row's chunk is ((db ^ (row & 3)) << 2) | x, so again only db << 6 is XORed per read.
__device__ __forceinline__ uint32_t v_lane_off(int lane) {
  const int i = lane & 15, qd = lane >> 4;
  const int rsub = i >> 2;                         // row inside the 4-row block == row & 3
  const int x = ((qd & 1) << 1) | ((i & 3) >> 1);  // 16-byte chunk inside the 64-byte column block
  return (uint32_t)((4 * (qd >> 1) + rsub) * ROW_BYTES + (rsub << 6) + (x << 4) + ((i & 1) << 3));
}
__device__ __forceinline__ bf16x8 read_v_frag(const char* v_lds, uint32_t lane_off, int j, int db) {
  const char* p0 = v_lds + (lane_off ^ (uint32_t)(db << 6)) + j * (16 * ROW_BYTES);
  const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)p0);
  const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0 + 8 * ROW_BYTES));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

template <int MB>
struct RowState {
  f32x16 o[4][MB];  // O^T accumulators: [depth block][row block], unnormalised
  float m[MB];      // running maximum of the scaled scores (log2 units), -inf before the first key
  float l[MB];      // this lane's share of the weight sum (the other half-wave holds the rest)
};

// Q as B operand: lane (row l%32 of block mb, half l/32) holds Q[row][ks*16 + 8*(l/32) .. +7].
template <int MB>
__device__ __forceinline__ void load_q(const Ctx& c, const DkEntry& e, int g, int row_base, int last_row, int lane,
                                       bf16x8 (&qf)[MB][8], int (&limit)[MB]) {
  const int gmask = (1 << c.gshift) - 1;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int row = min(row_base + mb * 32 + (lane & 31), last_row);
    const int tok = row >> c.gshift;
    const int head = (g << c.gshift) + (row & gmask);
    limit[mb] = e.n + tok;  // last visible absolute position (bottom-right causal alignment)
    const __bf16* qp = c.q + ((int64_t)(e.tok0 + tok) * c.n_q_heads + head) * D + 8 * (lane >> 5);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[mb][ks] = *(const bf16x8*)(qp + ks * 16);
  }
  // Make the compiler wait for Q here, once, instead of at first use inside the key loop, where its
  // vmcnt(0) would also drain the K/V tiles that are meant to stay in flight.
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(qf[mb][ks]));
}

// One K/V tile of KB*32 keys against MB*32 query rows: S^T, online softmax, O^T update.
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
template <int MB>
__device__ __forceinline__ void store_block(const Ctx& c, const DkEntry& e, const DkItem& it, int g, int row_local0,
                                            int lane, int db, const f32x16 (&o)[MB], const float (&ltot)[MB]) {
  const int h = lane >> 5;
  const int gmask = (1 << c.gshift) - 1;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int rl = row_local0 + mb * 32 + (lane & 31);
    if (rl >= it.nrows) continue;
    if (it.part_row0 >= 0) {
      float* p = c.parts + ((int64_t)(it.part_row0 + rl) * c.n_kv_heads + g) * PS + db * 32 + 4 * h;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        // PS is even, so every row starts 8-byte aligned: two float2 stores
        *(float2*)(p + 8 * r4) = make_float2(o[mb][4 * r4], o[mb][4 * r4 + 1]);
        *(float2*)(p + 8 * r4 + 2) = make_float2(o[mb][4 * r4 + 2], o[mb][4 * r4 + 3]);
      }
    } else {
      const int row = it.row0 + rl;
      const int tok = e.tok0 + (row >> c.gshift);
      const int head = (g << c.gshift) + (row & gmask);
      const float inv = 1.f / ltot[mb];
      __bf16* dst = c.out + ((int64_t)tok * c.n_q_heads + head) * D + db * 32 + 4 * h;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 v;
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = (__bf16)(o[mb][4 * r4 + t] * inv);
        *(bf16x4*)(dst + 8 * r4) = v;
      }
    }
  }
}

// Running maximum and weight sum of each row (partials) or the row's log-sum-exp (final output).
template <int MB>
__device__ __forceinline__ void store_ml(const Ctx& c, const DkEntry& e, const DkItem& it, int g, int row_local0,
                                         int lane, const float (&m)[MB], const float (&ltot)[MB]) {
  if (lane >= 32) return;
  const int gmask = (1 << c.gshift) - 1;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int rl = row_local0 + mb * 32 + lane;
    if (rl >= it.nrows) continue;
    if (it.part_row0 >= 0) {
      float* p = c.parts + ((int64_t)(it.part_row0 + rl) * c.n_kv_heads + g) * PS;
      p[D] = m[mb];
      p[D + 1] = ltot[mb];
    } else if (c.lse) {
      const int row = it.row0 + rl;
      const int tok = e.tok0 + (row >> c.gshift);
      const int head = (g << c.gshift) + (row & gmask);
      c.lse[(int64_t)tok * c.n_q_heads + head] = (m[mb] + __builtin_amdgcn_logf(ltot[mb])) * 0.6931471805599453f;
    }
  }
}

// ---- building blocks of the tile kernel's software pipeline -----------------------------------
// S^T of one 32-key block: 8 depth steps, MB row blocks.
template <int MB>
__device__ __forceinline__ void qk_block(const char* k_lds, int kb, const bf16x8 (&qf)[MB][8], f32x16 (&s)[MB],
                                         int lane) {
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) s[mb][r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const bf16x8 a = read_k_frag(k_lds, k_lane_off(lane), kb, ks);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[mb][ks], s[mb], 0, 0, 0);
  }
}

// Masks keys the row may not see (beyond the causal limit or past the end of a ragged tile).
template <int MB>
__device__ __forceinline__ void mask_block(f32x16 (&s)[MB], int kb, const int (&limit)[MB], int lane, int cnt,
                                           int pos) {
  const int h = lane >> 5;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int lim = min(cnt - 1, limit[mb] - pos);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
      if (key > lim) s[mb][r] = -INFINITY;
    }
  }
}

// Row maximum (scaled, log2 units) of one block, completed across the two half-waves.
template <int MB>
__device__ __forceinline__ void rowmax_block(const f32x16 (&s)[MB], float c, float (&mx)[MB]) {
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    float v = fmaxf(s[mb][0], s[mb][1]);
#pragma unroll
    for (int r = 2; r < 16; ++r) v = fmaxf(v, s[mb][r]);
    v = fmaxf(v, __shfl_xor(v, 32));
    mx[mb] = v * c;
  }
}

// The reference maximum only moves when some row's maximum grew by more than this (log2 units), so
// the rescale of O is rare once the first tiles have been seen; weights then stay below 2^8.
constexpr float RESCALE_SLACK = 8.f;

// x *= f for an accumulator that must stay in the AGPR half of the register file.  The O^T accumulators
// are only ever touched by MFMAs and by this (rare) rescale; going through an "a" constrained asm keeps
// the compiler from moving all 128 of them to VGPRs and back on every trip of the key loop.
__device__ __forceinline__ void scale_acc(float& x, float f) {
  float t;
  asm volatile(
      "v_accvgpr_read_b32 %1, %0\n\t"
      "v_mul_f32 %1, %1, %2\n\t"
      "v_accvgpr_write_b32 %0, %1"
      : "+a"(x), "=&v"(t)
      : "v"(f));
}

// Raises the reference maxima to cover mx and rescales O and l, if any row of the wavefront needs it.
template <int MB>
__device__ __forceinline__ void maybe_rescale(RowState<MB>& st, const float (&mx)[MB]) {
  bool grow = false;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) grow |= mx[mb] > st.m[mb] + RESCALE_SLACK;
  if (__builtin_amdgcn_ballot_w64(grow) == 0) return;
  // MFMA results must have left the matrix pipeline before the plain reads below (the compiler does not
  // look into the asm), and the writes must have landed before the next MFMA reads them: pad generously,
  // this path is rare.
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const float mn = fmaxf(st.m[mb], mx[mb]);
    const float ms = (mn == -INFINITY) ? 0.f : mn;
    const float alpha = __builtin_amdgcn_exp2f(st.m[mb] - ms);  // 1 for rows whose maximum did not move
    st.m[mb] = mn;
    st.l[mb] *= alpha;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float x = st.o[db][mb][r];
        scale_acc(x, alpha);
        st.o[db][mb][r] = x;
      }
  }
  asm volatile("s_nop 7" ::: "memory");
}

// Weights of one 32-key block against the current reference maxima, their sum, and the bf16 B operands.
template <int MB>
__device__ __forceinline__ void exp_block(f32x16 (&s)[MB], RowState<MB>& st, float c, bf16x8 (&pf)[MB][2]) {
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const float ms = (st.m[mb] == -INFINITY) ? 0.f : st.m[mb];
    float rs = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mb][r], c, -ms));
      rs += p;
      s[mb][r] = p;
    }
    st.l[mb] += rs;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < 8; ++t) pf[mb][j][t] = (__bf16)s[mb][8 * j + t];
  }
}

// O^T += V^T P^T for one 32-key block (two 16-key steps).
template <int MB>
__device__ __forceinline__ void pv_block(const char* v_lds, int kb, const bf16x8 (&pf)[MB][2], RowState<MB>& st,
                                         int lane) {
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const bf16x8 vf = read_v_frag(v_lds, v_lane_off(lane), 2 * kb + j, db);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        st.o[db][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[mb][j], st.o[db][mb], 0, 0, 0);
    }
}

// One 64-key tile: S^T of both 32-key blocks (sharing every Q operand), one maximum update for the
// tile, then weights and PV block by block, so the second block's exponentials can issue while the
// first block's PV MFMAs run.
template <int MB>
__device__ __forceinline__ void tile64(const char* k_lds, const char* v_lds, const bf16x8 (&qf)[MB][8],
                                       RowState<MB>& st, const int (&limit)[MB], float c, int lane, int cnt, int pos,
                                       bool need_mask) {
  f32x16 s0[MB], s1[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) s0[mb][r] = s1[mb][r] = 0.f;
  const uint32_t koff = k_lane_off(lane);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const bf16x8 a0 = read_k_frag(k_lds, koff, 0, ks);
    const bf16x8 a1 = read_k_frag(k_lds, koff, 1, ks);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      s0[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[mb][ks], s0[mb], 0, 0, 0);
      s1[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[mb][ks], s1[mb], 0, 0, 0);
    }
  }
  if (need_mask) {  // wave-uniform: only diagonal and ragged tiles take this path
    mask_block<MB>(s0, 0, limit, lane, cnt, pos);
    mask_block<MB>(s1, 1, limit, lane, cnt, pos);
  }
  float mx0[MB], mx1[MB];
  rowmax_block<MB>(s0, c, mx0);
  rowmax_block<MB>(s1, c, mx1);
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) mx0[mb] = fmaxf(mx0[mb], mx1[mb]);
  maybe_rescale<MB>(st, mx0);
  bf16x8 p[MB][2];
  exp_block<MB>(s0, st, c, p);
  pv_block<MB>(v_lds, 0, p, st, lane);
  exp_block<MB>(s1, st, c, p);
  pv_block<MB>(v_lds, 1, p, st, lane);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// ------------------------------------------------------------------------------------------------
// Tile kernel.  grid = items * n_kv_heads (KV head fastest, so the workgroups of one head share an
// XCD's L2 when there are 8 heads), block = 256.  LDS: 2 stages x (K 16 KiB + V 16 KiB).
// ------------------------------------------------------------------------------------------------
constexpr int TILE_KT = 64;
constexpr int TILE_STAGES = 3;
constexpr int TILE_STAGE_BYTES = 2 * TILE_KT * ROW_BYTES;
constexpr int TILE_LDS_BYTES = TILE_STAGES * TILE_STAGE_BYTES;

__global__ __launch_bounds__(256, 1) void attend_tile_kernel(Ctx c) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int MB = 2;
  const int g = blockIdx.x % c.n_kv_heads;
  const DkItem it = load_desc(c.items, blockIdx.x / c.n_kv_heads);
  const DkEntry e = load_desc(c.entries, it.entry);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int last_row = it.row0 + it.nrows - 1;
  const int wave_row0 = it.row0 + wave * (MB * 32);
  const bool wave_active = wave_row0 <= last_row;
  const int wave_min_limit = e.n + (min(wave_row0, last_row) >> c.gshift);
  const int wave_max_limit = e.n + (min(wave_row0 + MB * 32 - 1, last_row) >> c.gshift);

  bf16x8 qf[MB][8];
  int limit[MB];
  load_q<MB>(c, e, g, wave_row0, last_row, lane, qf, limit);

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

  // Three LDS stages, one barrier per tile.  Iteration t: wait for this wavefront's share of tile t,
  // barrier (every wavefront has also finished computing tile t-1, whose stage is therefore free),
  // start the loads of tile t+2 into that stage, compute tile t.
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
  KvTile t0, t1, t2;  // tile being computed, next, the one after
  bool have0 = cur.next(c, g, TILE_KT, t0);
  bool have1 = have0 && cur.next(c, g, TILE_KT, t1);
  if (have0) issue(t0, 0);
  if (have1) issue(t1, 1);
  int stage = 0;
  while (have0) {
    if (have1) wait_vmcnt<8>(); else wait_vmcnt<0>();  // tile t has landed; tile t+1 may still be in flight
    __builtin_amdgcn_s_barrier();
    const bool have2 = have1 && cur.next(c, g, TILE_KT, t2);
    if (have2) issue(t2, stage == 0 ? 2 : stage - 1);
    if (wave_active && t0.pos <= wave_max_limit) {
      const char* kl = smem + stage * TILE_STAGE_BYTES;
      const char* vl = kl + TILE_KT * ROW_BYTES;
      const bool need_mask = t0.cnt < TILE_KT || t0.pos + TILE_KT - 1 > wave_min_limit;
      tile64<MB>(kl, vl, qf, st, limit, c.c, lane, t0.cnt, t0.pos, need_mask);
    }
    t0 = t1;
    t1 = t2;
    have0 = have1;
    have1 = have2;
    stage = stage == 2 ? 0 : stage + 1;
  }

  float ltot[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) ltot[mb] = st.l[mb] + __shfl_xor(st.l[mb], 32);
  if (wave_active) {
#pragma unroll
    for (int db = 0; db < 4; ++db) store_block<MB>(c, e, it, g, wave * (MB * 32), lane, db, st.o[db], ltot);
    store_ml<MB>(c, e, it, g, wave * (MB * 32), lane, st.m, ltot);
  }
}

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

Ctx make_ctx(const AttendArgs& a, const DkItem* items) {
  Ctx c;
  c.entries = a.entries;
  c.segs = a.segs;
  c.items = items;
  c.q = (const __bf16*)a.q;
  c.k_arena = (const char*)a.arena.k_arena;
  c.v_arena = (const char*)a.arena.v_arena;
  c.k_new = (const char*)a.k_new;
  c.v_new = (const char*)a.v_new;
  c.out = (__bf16*)a.out;
  c.lse = a.lse;
  c.parts = a.parts;
  c.c = a.scale * 1.4426950408889634f;
  c.n_q_heads = a.arena.n_q_heads;
  c.n_kv_heads = a.arena.n_kv_heads;
  int group = a.arena.n_q_heads / a.arena.n_kv_heads, sh = 0;
  while ((1 << sh) < group) ++sh;
  c.gshift = sh;
  c.arena_cells = a.arena.arena_cells;
  return c;
}

}  // namespace

hipError_t launch_attend_tile(const AttendArgs& a, const DkItem* items, int32_t n_items, hipStream_t stream) {
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

hipError_t launch_attend_stream(const AttendArgs& a, const DkItem* items, int32_t n_items, hipStream_t stream) {
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
