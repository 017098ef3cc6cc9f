// Shared device code of the bf16 MFMA attention kernels (gfx950, head_dim 128): descriptor access,
// the walk over a slot's key segments, HBM -> LDS tile loads, MFMA operand reads and result stores.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace dk {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(3))) bf16x4* lds_bf16x4_ptr;
typedef __attribute__((address_space(1))) const void* glb_void_ptr;

constexpr int D = 128;
constexpr int ROW_BYTES = 256;
// Split partials: per (partial row, KV head) D unnormalised fp32 sums in `parts` (512-byte rows) and the pair
// (running maximum in log2 units, weight sum) in `parts_ml`.

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

// Kernel-argument form of the descriptor blob: the kernels take it as their FIRST argument, so in the inline
// instantiation it starts the kernel-argument segment and descriptor "pointers" are byte offsets from there.
template <bool INLINE> struct BlobArg;
template <> struct BlobArg<true> { InlineBlob blob; };
template <> struct BlobArg<false> { char unused; };

template <bool INLINE, typename T>
__device__ __forceinline__ const T* resolve_desc(const T* p) {
  if constexpr (INLINE) {
    typedef const __attribute__((address_space(4))) char* const_char_ptr;
    const_char_ptr base = (const_char_ptr)__builtin_amdgcn_kernarg_segment_ptr();
    return (const T*)((uintptr_t)base + (uintptr_t)p);
  } else {
    return p;
  }
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
  float* __restrict__ parts_ml;
  float c;  // softmax scale * log2(e): scores are handled in log2 units
  int32_t n_q_heads, n_kv_heads, gshift;
  int64_t arena_cells;
  const int32_t* cells;  // small append-and-attend calls: arena cell of every new token
  int32_t n_scatter;     // how many tokens this launch writes into the arena (0: none)
};

// A run of at most KT consecutive K/V rows, all inside one segment.
struct KvTile {
  const char* k;
  const char* v;
  uint32_t stride;  // bytes between consecutive rows
  int32_t cnt;      // valid rows (>= 1)
  int32_t pos;      // logical position of row 0
};

// Walks the logical key positions [p, hi) of an entry, segment by segment.  The state of the segment
// being walked (row pointers at position p, row stride, end position) is kept in a handful of scalars,
// so the common step touches neither the segment table nor the kernel arguments.
struct KvCursor {
  const DkSeg* segs;
  int32_t si, se, p, hi;
  int32_t seg_end = 0;  // first position past the current segment (0: no segment loaded yet)
  const char* k = nullptr;
  const char* v = nullptr;
  uint32_t stride = 0;

  __device__ __forceinline__ void enter_segment(const Ctx& c, int g) {
    DkSeg s = load_desc(segs, si);
    while (s.pos + s.len <= p && si + 1 < se) s = load_desc(segs, ++si);
    const int32_t off = p - s.pos;
    seg_end = s.pos + s.len;
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
  }

  __device__ __forceinline__ bool next(const Ctx& c, int g, int kt, KvTile& t) {
    if (p >= hi) return false;
    if (p >= seg_end) enter_segment(c, g);
    t.cnt = min(kt, min(seg_end, hi) - p);
    t.k = k;
    t.v = v;
    t.stride = stride;
    t.pos = p;
    p += t.cnt;
    const uint32_t adv = (uint32_t)t.cnt * stride;
    k += adv;
    v += adv;
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

// Issues the loads of a wavefront's Q fragments; wait_q() below is where they must have arrived.  What is
// put between the two (finding the first K/V tiles and requesting them) overlaps with the Q round trip.
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
}

// Makes the compiler wait for Q here, once, instead of at first use inside the key loop, where its
// vmcnt(0) would also drain the K/V tiles that are meant to stay in flight.  (The wait it emits here is a
// vmcnt(0) as well: K/V tiles requested before this point land before the key loop starts.)
template <int MB>
__device__ __forceinline__ void wait_q(const bf16x8 (&qf)[MB][8]) {
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(qf[mb][ks]));
}

// One K/V tile of KB*32 keys against MB*32 query rows: S^T, online softmax, O^T update.
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
      float* p = c.parts + ((int64_t)(it.part_row0 + rl) * c.n_kv_heads + g) * D + db * 32 + 4 * h;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *(f32x4*)(p + 8 * r4) = f32x4{o[mb][4 * r4], o[mb][4 * r4 + 1], o[mb][4 * r4 + 2], o[mb][4 * r4 + 3]};
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

// The same store through a private LDS staging area of 8 KiB, so that every store instruction of the wavefront
// writes eight whole 128-byte pieces of eight rows instead of 64 scattered 8-byte pieces: the accumulator
// layout (lane = row) is turned into (8 lanes = 128 bytes of one row) on the way.  16-byte chunks of a staged
// row are XOR-swizzled with the row number, which keeps both the writes (one row per lane) and the reads
// (eight lanes per row) free of bank conflicts.  Covers 64 rows x all 128 depths: four passes of one depth
// block for fp32 partials, two passes of two depth blocks for the bf16 output.  LDS operations of one
// wavefront execute in order, so no wait is needed between a pass's writes and reads or between passes.
template <int MB>
__device__ __forceinline__ void store_rows_staged(const Ctx& c, const DkEntry& e, const DkItem& it, int g,
                                                  int row_local0, int lane, char* stage, const f32x16 (&o)[4][MB],
                                                  const float (&ltot)[MB]) {
  static_assert(MB == 2, "64 rows per wavefront");
  const int h = lane >> 5, r = lane & 31;
  const int rd_row = lane >> 3, rd_chunk = lane & 7;  // reader: row inside a group of eight, 16-byte chunk
  const int gmask = (1 << c.gshift) - 1;
  if (it.part_row0 >= 0) {
#pragma unroll
    for (int db = 0; db < 4; ++db) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int R = mb * 32 + r;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *(f32x4*)(stage + R * 128 + (((2 * r4 + h) ^ (R & 7)) << 4)) =
              f32x4{o[db][mb][4 * r4], o[db][mb][4 * r4 + 1], o[db][mb][4 * r4 + 2], o[db][mb][4 * r4 + 3]};
      }
#pragma unroll
      for (int ps = 0; ps < 8; ++ps) {
        const int R = ps * 8 + rd_row;
        const f32x4 v = *(const f32x4*)(stage + R * 128 + ((rd_chunk ^ (R & 7)) << 4));
        const int rl = row_local0 + R;
        if (rl < it.nrows)
          *(f32x4*)(c.parts + ((int64_t)(it.part_row0 + rl) * c.n_kv_heads + g) * D + db * 32 + rd_chunk * 4) = v;
      }
      __builtin_amdgcn_sched_barrier(0);  // one pass at a time: keeps the passes' registers from piling up
    }
  } else {
    float inv[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) inv[mb] = 1.f / ltot[mb];
#pragma unroll
    for (int dp = 0; dp < 2; ++dp) {  // depth blocks 2 dp and 2 dp + 1: 64 bf16 = 128 bytes per row
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int R = mb * 32 + r;
#pragma unroll
        for (int d2 = 0; d2 < 2; ++d2)
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            bf16x4 v;
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] = (__bf16)(o[2 * dp + d2][mb][4 * r4 + t] * inv[mb]);
            // bf16 columns d2*32 + 8*r4 + 4h .. +3: 8-byte piece (8*d2 + 2*r4 + h) of the 128-byte row
            const int piece = 8 * d2 + 2 * r4 + h;
            *(bf16x4*)(stage + R * 128 + ((((piece >> 1) ^ (R & 7)) << 4) | ((piece & 1) << 3))) = v;
          }
      }
#pragma unroll
      for (int ps = 0; ps < 8; ++ps) {
        const int R = ps * 8 + rd_row;
        const bf16x8 v = *(const bf16x8*)(stage + R * 128 + ((rd_chunk ^ (R & 7)) << 4));
        const int rl = row_local0 + R;
        if (rl < it.nrows) {
          const int row = it.row0 + rl;
          const int tok = e.tok0 + (row >> c.gshift);
          const int head = (g << c.gshift) + (row & gmask);
          *(bf16x8*)(c.out + ((int64_t)tok * c.n_q_heads + head) * D + dp * 64 + rd_chunk * 8) = v;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
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
      float* p = c.parts_ml + ((int64_t)(it.part_row0 + rl) * c.n_kv_heads + g) * 2;
      *(float2*)p = make_float2(m[mb], ltot[mb]);
    } else if (c.lse) {
      const int row = it.row0 + rl;
      const int tok = e.tok0 + (row >> c.gshift);
      const int head = (g << c.gshift) + (row & gmask);
      c.lse[(int64_t)tok * c.n_q_heads + head] = (m[mb] + __builtin_amdgcn_logf(ltot[mb])) * 0.6931471805599453f;
    }
  }
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Append-and-attend calls small enough for their descriptors to travel in the kernel arguments: the attention
// kernel also writes the call's new K/V rows (token-major, as staged in k_new / v_new) into their arena cells, so
// that no separate copy kernel has to be launched.  The cells are fresh ones that no attention work of this launch
// reads (the new tokens are attended from the staged rows), so the order against the rest of the kernel is free:
// every workgroup copies an equal run right after its first K/V requests, whose latency covers the copy's.
// The copy is cut into 16-byte pieces, piece p = (token, K or V, KV head, position in the row); a thread has four
// loads in flight before its first store.
template <bool INLINE>
__device__ __forceinline__ void scatter_new_rows(const Ctx& c) {
  if (c.n_scatter <= 0) return;
  const int32_t* cells = resolve_desc<INLINE>(c.cells);
  const int vecs = c.n_kv_heads * (ROW_BYTES / 16);  // pieces of one token's K (as many for V)
  const int total = c.n_scatter * 2 * vecs;
  const int per = ((total + (int)gridDim.x - 1) / (int)gridDim.x + 255) & ~255;
  const int begin = min(total, (int)blockIdx.x * per), end = min(total, begin + per);
  const auto locate = [&](int p, const char*& src, char*& dst) {
    p = min(p, end - 1);  // (threads past the end repeat the last piece: same bytes)
    const int t = p / (2 * vecs), r = p - t * (2 * vecs);
    const bool is_v = r >= vecs;
    const int j = is_v ? r - vecs : r;
    const int g = j / (ROW_BYTES / 16), piece = j % (ROW_BYTES / 16);
    const int64_t cell = cells[t];
    src = (is_v ? c.v_new : c.k_new) + ((int64_t)t * c.n_kv_heads + g) * ROW_BYTES + piece * 16;
    dst = const_cast<char*>(is_v ? c.v_arena : c.k_arena) + ((int64_t)g * c.arena_cells + cell) * ROW_BYTES + piece * 16;
  };
  for (int base = begin + (int)threadIdx.x; base < end; base += 4 * 256) {
    const char *s0, *s1, *s2, *s3;
    char *d0, *d1, *d2, *d3;
    locate(base, s0, d0);
    locate(base + 256, s1, d1);
    locate(base + 512, s2, d2);
    locate(base + 768, s3, d3);
    const uint4 v0 = *(const uint4*)s0, v1 = *(const uint4*)s1, v2 = *(const uint4*)s2, v3 = *(const uint4*)s3;
    *(uint4*)d0 = v0;
    *(uint4*)d1 = v1;
    *(uint4*)d2 = v2;
    *(uint4*)d3 = v3;
  }
}

inline Ctx make_ctx(const AttendArgs& a, const DkItem* items) {
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
  c.parts_ml = a.parts_ml;
  c.c = a.scale * 1.4426950408889634f;
  c.n_q_heads = a.arena.n_q_heads;
  c.n_kv_heads = a.arena.n_kv_heads;
  int group = a.arena.n_q_heads / a.arena.n_kv_heads, sh = 0;
  while ((1 << sh) < group) ++sh;
  c.gshift = sh;
  c.arena_cells = a.arena.arena_cells;
  c.cells = a.cells;
  c.n_scatter = a.scatter ? a.total_tokens : 0;
  return c;
}

}  // namespace mfma
}  // namespace dk
