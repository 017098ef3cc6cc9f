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
//   stream kernel  small Delta (G*Delta <= 96): every wavefront streams its own slice of the keys
//                  through private LDS stages with no barriers, the four states are merged at the
//                  end (HBM bound)
//
// K/V tiles go HBM -> LDS with global_load_lds_dwordx4 (no VGPR staging).  Rows are 256 B; the 16-byte
// chunks of a row are XOR-swizzled so that the K reads (ds_read_b128, one row per lane) and the V
// reads (ds_read_b64_tr_b16, 4 rows x 16 columns per 16 lanes) are bank-conflict free.
#include <hip/hip_runtime.h>

#include <mutex>

#include "attend_common.hpp"
#include "kernels.hpp"

namespace dk {
namespace mfma {

#ifdef DK_TRACE  // timeline build: wall-clock stamps (100 MHz) per workgroup and unit
__device__ unsigned long long g_strace[256][8][12];
#define DK_STR(seq, ph)                                                                                      \
  do {                                                                                                       \
    if (lane == 0 && (seq) < 8 && blockIdx.x < 256) g_strace[blockIdx.x][(seq)][(ph)] = wall_clock64();       \
  } while (0)
#else
#define DK_STR(seq, ph)
#endif

template <int MB>
struct RowState {
  f32x16 o[4][MB];  // O^T accumulators: [depth block][row block], unnormalised
  float m[MB];      // running maximum of the scaled scores (log2 units), -inf before the first key
  float l[MB];      // this lane's share of the weight sum (the other half-wave holds the rest)
};

// All MFMA operand fragments of one 32-key tile, read out of its LDS stage in one go: once they are in
// registers the stage can take the next HBM load while the tile is still being computed.
struct TileFrags {
  bf16x8 k[8];     // [depth step]
  bf16x8 v[2][4];  // [key step][depth block]
};
__device__ __forceinline__ void read_frags(const char* k_lds, const char* v_lds, int lane, TileFrags& f) {
  const uint32_t koff = k_lane_off(lane), voff = v_lane_off(lane);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) f.k[ks] = read_k_frag(k_lds, koff, 0, ks);
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int db = 0; db < 4; ++db) f.v[j][db] = read_v_frag(v_lds, voff, j, db);
}

constexpr float STREAM_RESCALE_SLACK = 8.f;  // log2 units, as in the tile kernel

__device__ __forceinline__ float stream_max3(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}

// O *= alpha for one accumulator, written so that the accumulators stay in the accumulation registers: with plain
// C++ here the compiler keeps a second copy of all of O in ordinary registers, refreshed for every tile (one
// v_accvgpr_read per element and tile) only to serve this rarely taken path.  Every MFMA that wrote O has retired
// by the time this runs: the scores of the current tile, produced by later MFMAs, have already been read.
__device__ __forceinline__ float scale_acc(float o, float alpha) {
  float t;
  asm volatile(
      "v_accvgpr_read_b32 %1, %0\n\t"
      "s_nop 0\n\t"
      "v_mul_f32 %1, %1, %2\n\t"
      "s_nop 0\n\t"
      "v_accvgpr_write_b32 %0, %1"
      : "+a"(o), "=&v"(t)
      : "v"(alpha));
  return o;
}

// Q as B operand: lane (row l%32 of block mb, half l/32) holds Q[row][ks*16 + 8*(l/32) .. +7].  With one or two
// row blocks the unit's Q fragments stay in registers for the whole unit; with three (96 registers next to 192
// of accumulators) they would not fit, so each tile reads them from the Q area in LDS again (24 ds_read_b128 per
// tile next to the tile's own 16: LDS bandwidth is idle here).
template <int MB>
struct QFrags {
  static constexpr bool IN_LDS = MB > 2;
  bf16x8 r[IN_LDS ? 1 : MB][8];
  const char* q_lds;
  uint32_t koff;
  __device__ __forceinline__ void load() {
    if constexpr (!IN_LDS) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) r[mb][ks] = read_k_frag(q_lds, koff, mb, ks);
    }
  }
  __device__ __forceinline__ bf16x8 get(int mb, int ks) const {
    if constexpr (IN_LDS) return read_k_frag(q_lds, koff, mb, ks);
    else return r[mb][ks];
  }
};

// One 32-key tile against MB*32 query rows, operands in registers: S^T, online softmax, O^T update.
template <int MB>
__device__ __forceinline__ void compute_tile(const TileFrags& f, const QFrags<MB>& qf, RowState<MB>& st,
                                             const int (&limit)[MB], float c, int lane, int cnt, int pos,
                                             bool need_mask) {
  const int h = lane >> 5;
  bf16x8 pf[MB][2];
  f32x16 s[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) s[mb][r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.k[ks], qf.get(mb, ks), s[mb], 0, 0, 0);

  if (need_mask) {
    // accumulator r is key 8*(r/4) + 4h + r%4 of the tile
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int lim = min(cnt - 1, limit[mb] - pos);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = 8 * (r >> 2) + 4 * h + (r & 3);
        if (key > lim) s[mb][r] = -INFINITY;
      }
    }
  }

  // row maxima; the reference maximum of a row is only raised (and O, l rescaled) when the tile outgrows
  // it by more than the slack, so after the first tiles the 128 multiplies on O are rare
  float mx[MB];
  bool grow = false;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    float v = stream_max3(s[mb][0], s[mb][1], s[mb][2]);
#pragma unroll
    for (int r = 3; r < 15; r += 2) v = stream_max3(v, s[mb][r], s[mb][r + 1]);
    v = fmaxf(v, s[mb][15]);
    v = fmaxf(v, __shfl_xor(v, 32));
    mx[mb] = v * c;
    grow |= mx[mb] > st.m[mb] + STREAM_RESCALE_SLACK;
  }
  if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const float mn = fmaxf(st.m[mb], mx[mb]);
      const float mz = (mn == -INFINITY) ? 0.f : mn;  // every key so far masked: keep the arithmetic finite
      const float alpha = __builtin_amdgcn_exp2f(st.m[mb] - mz);
      st.m[mb] = mn;
      st.l[mb] *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[db][mb][r] = scale_acc(st.o[db][mb][r], alpha);
    }
  }

#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const float ms = (st.m[mb] == -INFINITY) ? 0.f : st.m[mb];
    float rs[2] = {0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mb][8 * j + 2 * w], c, -ms));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mb][8 * j + 2 * w + 1], c, -ms));
        rs[(j * 4 + w) & 1] += p0 + p1;  // (no v_dot2 here: the dot instructions queue behind the MFMAs)
        pf[mb][j][2 * w] = (__bf16)p0;
        pf[mb][j][2 * w + 1] = (__bf16)p1;
      }
    st.l[mb] += rs[0] + rs[1];
  }

#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        st.o[db][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v[j][db], pf[mb][j], st.o[db][mb], 0, 0, 0);
}

// Accumulator r of depth block db is depth db*32 + 8*(r/4) + 4h + r%4: four consecutive depths per r/4.
// ------------------------------------------------------------------------------------------------
// Stream kernel.  grid = chains, block = 256.  A workgroup walks a chain of units (item, KV head).  Each
// wavefront owns a quarter of the unit's key range and two private 32-key stages (K 8 KiB + V 8 KiB
// each); no barrier in the key loop.  At the end of a unit the four (O, m, l) states are merged through
// LDS, wavefront w finishing depth block w.
//
// Unit changes.  The merge buffer is the wavefronts' second stages only, one row block at a time, so that a
// wavefront that has finished its quarter can at once request the next unit's first K/V tile into its first
// stage; the next unit's Q rows are requested into an LDS area of their own right after the first merge
// barrier (no wavefront reads the current Q any more then), and the second tile as soon as the merge buffer
// has been read.  The merge thus runs under the latency of those requests instead of in front of it.
//
// Which unit comes next.  Small launches (descriptors in the kernel arguments) walk the chains the planner linked.
// Otherwise the units form one queue, longest first: workgroup w starts with unit w and every further unit is
// drawn from a counter in device memory (uploaded with the descriptors, starting at the number of workgroups) by
// one atomic add.  The compute units do not stream equally fast -- by 10 % and more between XCDs, differently from
// box to box and batch to batch -- so chains of equal length planned on the host end up to 25 % apart; with the
// queue a faster workgroup simply takes the next unit earlier.  Wavefront 0 draws half-way through its share of
// the current unit (the order of drawing is the order of finishing, and the round trip is hidden), fetches the
// drawn unit's descriptors and hands them to the other wavefronts through LDS at the unit's end.  Which workgroup
// computes a unit has no influence on the unit's result.
//
// LDS map: [0, 128 KiB) stages, wavefront w at w * 32 KiB (stage 0, stage 1); then the (m, l) exchange
// (2 KiB); then the Q rows of the unit, laid out and swizzled like a K tile of MB * 32 rows; then the next
// unit's descriptors as published by wavefront 0.
// ------------------------------------------------------------------------------------------------
constexpr int STREAM_KT = 32;
constexpr int STREAM_STAGE_BYTES = 2 * STREAM_KT * ROW_BYTES;  // 16 KiB
constexpr int STREAM_WAVE_BYTES = 2 * STREAM_STAGE_BYTES;      // 32 KiB
constexpr int STREAM_ML_OFFSET = 4 * STREAM_WAVE_BYTES;        // after the stages
constexpr int STREAM_MAX_MB = 3;                               // row blocks of the widest instantiation
constexpr int STREAM_ML_ROWS = STREAM_MAX_MB * 32;             // rows per wavefront in the (m, l) exchange
constexpr int STREAM_Q_OFFSET = STREAM_ML_OFFSET + 4 * STREAM_ML_ROWS * 2 * 4;
constexpr int STREAM_NEXT_OFFSET = STREAM_Q_OFFSET + STREAM_MAX_MB * 32 * ROW_BYTES;
constexpr int STREAM_LDS_BYTES = STREAM_NEXT_OFFSET + 128;
static_assert(STREAM_LDS_BYTES <= 160 * 1024, "one workgroup per compute unit: all of its LDS, no more");

// One wavefront moves 4 query rows (1 KiB) HBM -> LDS into the Q area: packed row `blk * 4 + l / 16` of the
// unit (clamped to its last row), chunk slots swizzled as for a K tile so that read_k_frag serves as the
// reader of Q's B-operand fragments.  Every wavefront requests all rows itself: each only depends on its own
// requests, and the four write the same bytes.
__device__ __forceinline__ void load_q_rows4(const Ctx& c, const char* q_tok0, int g, int row0, int last_row,
                                             char* q_lds, int blk, int lane) {
  const int row = blk * 4 + (lane >> 4);
  const int slot = lane & 15;
  const int chunk = slot ^ (row & 15);
  const int arow = min(row0 + row, last_row);
  const int gmask = (1 << c.gshift) - 1;
  const uint32_t voff =
      (uint32_t)(((arow >> c.gshift) * c.n_q_heads + (g << c.gshift) + (arow & gmask)) * ROW_BYTES + chunk * 16);
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_void_ptr)(q_lds + blk * 1024);
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_addr), "v"(voff), "s"(q_tok0)
      : "memory", "m0");
}

__device__ __forceinline__ void lds_barrier() {
  // LDS traffic of this wavefront has completed; K/V requests stay in flight (no vmcnt wait here)
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// MB = 32-row blocks per unit: 1 when no unit of the launch has more than 32 packed rows (Delta <= 32 / G:
// decode and short verify steps then skip the all-padding blocks), 2 up to 64 rows, else 3 (up to 96 rows: between
// 64 and 96 rows a unit is still far below the MFMA/HBM ridge, and the tile kernel, built for 256-row tiles, keeps
// too little in flight to stream it well).
// INLINE: the descriptors arrive inside the kernel arguments (first argument) and the descriptor pointers are byte
// offsets into them; otherwise they point into the uploaded workspace.
template <int MB, bool INLINE>
__global__ __launch_bounds__(256, 1) void attend_stream_kernel(BlobArg<INLINE> blob, Ctx c, const int32_t* links,
                                                               int n_chains, int32_t* queue, int n_units) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  (void)blob;
  c.entries = resolve_desc<INLINE>(c.entries);
  c.segs = resolve_desc<INLINE>(c.segs);
  c.items = resolve_desc<INLINE>(c.items);
  links = resolve_desc<INLINE>(links);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* my = smem + wave * STREAM_WAVE_BYTES;
  float* ml = (float*)(smem + STREAM_ML_OFFSET);  // [wave][row 0..95][m, l]
  char* q_lds = smem + STREAM_Q_OFFSET;
  int32_t* next_lds = (int32_t*)(smem + STREAM_NEXT_OFFSET);  // [0] unit, [4..11] its DkItem, [12..19] its DkEntry
  const uint32_t koff = k_lane_off(lane);
  const bool queued = !INLINE && queue != nullptr;  // units are drawn from the queue (else: the planner's chains)
  int trace_seq = 0;
  (void)trace_seq;

  // ---- the unit being streamed, and the requests that open a unit ----------------------------------
  int unit = queued ? (int)blockIdx.x : load_desc(links, blockIdx.x);
  DkItem it = load_desc(c.items, unit / c.n_kv_heads);
  DkEntry e = load_desc(c.entries, it.entry);
  int g = unit % c.n_kv_heads;
  KvCursor cur{c.segs, 0, 0, 0, 0};
  KvTile t0, t1, t2;  // being computed, next, the one after
  bool have0 = false, have1 = false;

  auto issue = [&](const KvTile& t, int stage) {
    char* kl = my + stage * STREAM_STAGE_BYTES;
    char* vl = kl + STREAM_KT * ROW_BYTES;
#pragma unroll
    for (int b = 0; b < 8; ++b) load_rows4<false>(t.k, t.stride, t.cnt, kl, b, lane);
#pragma unroll
    for (int b = 0; b < 8; ++b) load_rows4<true>(t.v, t.stride, t.cnt, vl, b, lane);
  };
  // this wavefront's quarter of the unit's keys: cursor, first tile requested into stage 0
  auto open_keys = [&](const DkItem& u, const DkEntry& ue, int ug) {
    const int ntile = (u.kv_hi - u.kv_lo + STREAM_KT - 1) / STREAM_KT;
    const int per = (ntile + 3) / 4 * STREAM_KT;
    const int lo = min(u.kv_hi, u.kv_lo + wave * per);
    const int hi = min(u.kv_hi, lo + per);
    cur = KvCursor{c.segs, ue.seg_begin, ue.seg_end, lo, hi};
    have0 = cur.next(c, ug, STREAM_KT, t0);
    if (have0) issue(t0, 0);
  };
  auto open_q = [&](const DkItem& u, const DkEntry& ue, int ug) {
    const char* q_tok0 = (const char*)c.q + (int64_t)ue.tok0 * c.n_q_heads * ROW_BYTES;
#pragma unroll
    for (int b = 0; b < MB * 8; ++b) load_q_rows4(c, q_tok0, ug, u.row0, u.row0 + u.nrows - 1, q_lds, b, lane);
  };
  auto open_second = [&](int ug) {
    have1 = have0 && cur.next(c, ug, STREAM_KT, t1);
    if (have1) issue(t1, 1);
  };

  open_keys(it, e, g);
  open_q(it, e, g);
  open_second(g);
  if (wave == 0) DK_STR(0, 10);  // (kernel entry, a few scalar loads late)
  // small append-and-attend calls: this workgroup's share of the new rows goes into the arena now, under the
  // latency of the first unit's requests
  scatter_new_rows<INLINE>(c);

  while (true) {
    // The descriptors of the next unit are fetched while this one is being streamed, so that a unit change
    // does not start with a chain of dependent memory round trips.
    int next_unit = -1;
    DkItem next_it = it;
    DkEntry next_e = e;
    if (!queued) {
      next_unit = load_desc(links, n_chains + unit);
      if (next_unit >= 0) {
        next_it = load_desc(c.items, next_unit / c.n_kv_heads);
        next_e = load_desc(c.entries, next_it.entry);
      }
    }
    // queue: wavefront 0 draws in iteration draw_at of its key loop (an ordinary atomic: the compiler keeps account
    // of it and waits for the answer where it is first used, after the loop, when no K/V request is in flight)
    const bool drawer = queued && wave == 0;
    int drawn = 0;
    bool drew = false;
    const auto draw = [&]() {
      if (lane == 0) drawn = __hip_atomic_fetch_add(queue, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      drew = true;
    };
    const int last_row = it.row0 + it.nrows - 1;
    const int min_limit = e.n + (it.row0 >> c.gshift);

    RowState<MB> st;
    int limit[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      st.m[mb] = -INFINITY;
      st.l[mb] = 0.f;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[db][mb][r] = 0.f;
      limit[mb] = e.n + (min(it.row0 + mb * 32 + (lane & 31), last_row) >> c.gshift);
    }

    // Everything requested before the second tile has arrived: the unit's Q rows and its first tile.
    if (wave == 0) DK_STR(trace_seq, 0);
    if (have1) wait_vmcnt<16>(); else wait_vmcnt<0>();
    QFrags<MB> qf;
    qf.q_lds = q_lds;
    qf.koff = koff;
    qf.load();
    if (wave == 0) DK_STR(trace_seq, 1);

    // Two private stages per wavefront.  A tile's fragments are read into registers as soon as it has
    // landed and its stage is handed to the load of the tile after next at once, so two tiles (32 KiB per
    // wavefront) are in flight while one is being computed -- with only the other stage loading, HBM
    // latency would not be covered.
    int stage = 0;
    TileFrags fr;
    // (wavefront 0's share of the unit is at least this many tiles: ragged segment ends only add some)
    const int my_tiles = ((it.kv_hi - it.kv_lo + STREAM_KT - 1) / STREAM_KT + 3) / 4;
    const int draw_at = my_tiles / 2;
    int iter = 0;
    while (have0) {
      if (have1) wait_vmcnt<16>(); else wait_vmcnt<0>();
      const char* kl = my + stage * STREAM_STAGE_BYTES;
      read_frags(kl, kl + STREAM_KT * ROW_BYTES, lane, fr);
      const bool have2 = have1 && cur.next(c, g, STREAM_KT, t2);
      if (drawer && !drew && iter >= draw_at) draw();
      ++iter;
      if (have2) {
        // the stage may only be overwritten once every fragment read has returned
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        issue(t2, stage);
      }
      const bool need_mask = t0.cnt < STREAM_KT || t0.pos + STREAM_KT - 1 > min_limit;
      compute_tile<MB>(fr, qf, st, limit, c.c, lane, t0.cnt, t0.pos, need_mask);
      t0 = t1;
      t1 = t2;
      have0 = have1;
      have1 = have2;
      stage ^= 1;
    }
    DK_STR(trace_seq, 2 + wave);  // each wavefront's own end of streaming

    // ---- unit change: both stages of this wavefront are free ----------------------------------------
    if (drawer) {
      if (!drew) draw();  // (a share with no tiles at all)
      const int q = __builtin_amdgcn_readfirstlane(drawn);
      next_unit = q < n_units ? q : -1;
      if (next_unit >= 0) {
        next_it = load_desc(c.items, next_unit / c.n_kv_heads);
        next_e = load_desc(c.entries, next_it.entry);
      }
      if (lane == 0) {
        next_lds[0] = next_unit;
        next_lds[4] = next_it.entry;
        next_lds[5] = next_it.row0;
        next_lds[6] = next_it.nrows;
        next_lds[7] = next_it.kv_lo;
        next_lds[8] = next_it.kv_hi;
        next_lds[9] = next_it.part_row0;
        next_lds[12] = next_e.seg_begin;
        next_lds[13] = next_e.seg_end;
        next_lds[14] = next_e.n;
        next_lds[15] = next_e.delta;
        next_lds[16] = next_e.tok0;
      }
    }

    // ---- merge the four wavefront states ------------------------------------------------------------
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const float lt = st.l[mb] + __shfl_xor(st.l[mb], 32);
      if (lane < 32) {
        ml[(wave * STREAM_ML_ROWS + mb * 32 + lane) * 2] = st.m[mb];
        ml[(wave * STREAM_ML_ROWS + mb * 32 + lane) * 2 + 1] = lt;
      }
    }
    int next_g = 0;
    const int db = wave;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      // row block mb of every wavefront's O goes through the wavefronts' second stages: [db][r][lane]
      float* mine = (float*)(my + STREAM_STAGE_BYTES);
#pragma unroll
      for (int d4 = 0; d4 < 4; ++d4)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[(d4 * 16 + r) * 64 + lane] = st.o[d4][mb][r];
      lds_barrier();
      if (mb == 0) {
        if (wave == 0) DK_STR(trace_seq, 6);
        if (queued) {  // what wavefront 0 drew (field by field: the values must stay in scalar registers)
          const auto word = [&](int i) { return __builtin_amdgcn_readfirstlane(next_lds[i]); };
          next_unit = word(0);
          next_it.entry = word(4);
          next_it.row0 = word(5);
          next_it.nrows = word(6);
          next_it.kv_lo = word(7);
          next_it.kv_hi = word(8);
          next_it.part_row0 = word(9);
          next_e.seg_begin = word(12);
          next_e.seg_end = word(13);
          next_e.n = word(14);
          next_e.delta = word(15);
          next_e.tok0 = word(16);
        }
        next_g = next_unit % c.n_kv_heads;
        // every wavefront is past its key loop: its first stage may take the next unit's first tile, and no
        // wavefront reads the current unit's Q any more
        if (next_unit >= 0) {
          open_keys(next_it, next_e, next_g);  // (have0, t0, cur now belong to the next unit)
          open_q(next_it, next_e, next_g);
        }
      }
      const int row = mb * 32 + (lane & 31);
      float mw[4], lw[4];
      float mx = -INFINITY;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        mw[w] = ml[(w * STREAM_ML_ROWS + row) * 2];
        lw[w] = ml[(w * STREAM_ML_ROWS + row) * 2 + 1];
        mx = fmaxf(mx, mw[w]);
      }
      const float ms = (mx == -INFINITY) ? 0.f : mx;
      float lsum = 0.f;
      f32x16 acc[1];
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[0][r] = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float f = __builtin_amdgcn_exp2f(mw[w] - ms);
        lsum += f * lw[w];
        const float* theirs = (const float*)(smem + w * STREAM_WAVE_BYTES + STREAM_STAGE_BYTES);
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][r] += f * theirs[(db * 16 + r) * 64 + lane];
      }
      // the buffer has been read everywhere: the next row block, or the next unit's second tile, may overwrite it
      if (mb + 1 < MB || next_unit >= 0) lds_barrier();
      // (one row block's result at a time: the merged rows of all blocks together would not fit the registers)
      const float mm[1] = {mx}, ll[1] = {lsum};
      store_block<1>(c, e, it, g, mb * 32, lane, db, acc, ll);
      if (wave == 0) store_ml<1>(c, e, it, g, mb * 32, lane, mm, ll);
    }
    // (after the stores: the wait that opens the next unit lets exactly this request stay in flight)
    if (next_unit >= 0) open_second(next_g);
    if (wave == 0) DK_STR(trace_seq, 7);
#ifdef DK_TRACE
    if (threadIdx.x == 0 && trace_seq < 8 && blockIdx.x < 256) g_strace[blockIdx.x][trace_seq][8] = (unsigned long long)(it.kv_hi - it.kv_lo);
    ++trace_seq;
#endif
    if (next_unit < 0) break;
    unit = next_unit;
    it = next_it;
    e = next_e;
    g = next_g;
  }
}

}  // namespace mfma

hipError_t launch_attend_stream(const AttendArgs& a, const DkItem* items, const int32_t* links, int32_t n_chains,
                                int32_t max_rows, int32_t* queue, int32_t n_units, hipStream_t stream) {
  using namespace mfma;
  if (n_chains <= 0) return hipSuccess;
  if (a.arena.head_dim != D || a.arena.dtype != 1 || max_rows > STREAM_MAX_MB * 32) return hipErrorInvalidValue;
  if (queue && a.inline_blob) return hipErrorInvalidValue;  // the queue's counter needs device memory
  // once per process, whatever thread or pool gets here first
  static std::once_flag attr_once;
  static hipError_t attr_status = hipSuccess;
  std::call_once(attr_once, [] {
    const void* kernels[6] = {(const void*)attend_stream_kernel<1, false>, (const void*)attend_stream_kernel<1, true>,
                              (const void*)attend_stream_kernel<2, false>, (const void*)attend_stream_kernel<2, true>,
                              (const void*)attend_stream_kernel<3, false>, (const void*)attend_stream_kernel<3, true>};
    for (const void* k : kernels)
      if (attr_status == hipSuccess)
        attr_status = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, STREAM_LDS_BYTES);
  });
  if (attr_status != hipSuccess) return attr_status;
  const Ctx c = make_ctx(a, items);
  const dim3 grid((unsigned)n_chains);
  if (a.inline_blob) {
    BlobArg<true> blob{*a.inline_blob};
    if (max_rows <= 32) attend_stream_kernel<1, true><<<grid, 256, STREAM_LDS_BYTES, stream>>>(blob, c, links, n_chains, queue, n_units);
    else if (max_rows <= 64) attend_stream_kernel<2, true><<<grid, 256, STREAM_LDS_BYTES, stream>>>(blob, c, links, n_chains, queue, n_units);
    else attend_stream_kernel<3, true><<<grid, 256, STREAM_LDS_BYTES, stream>>>(blob, c, links, n_chains, queue, n_units);
  } else {
    const BlobArg<false> none{0};
    if (max_rows <= 32) attend_stream_kernel<1, false><<<grid, 256, STREAM_LDS_BYTES, stream>>>(none, c, links, n_chains, queue, n_units);
    else if (max_rows <= 64) attend_stream_kernel<2, false><<<grid, 256, STREAM_LDS_BYTES, stream>>>(none, c, links, n_chains, queue, n_units);
    else attend_stream_kernel<3, false><<<grid, 256, STREAM_LDS_BYTES, stream>>>(none, c, links, n_chains, queue, n_units);
  }
  return hipGetLastError();
}

}  // namespace dk
