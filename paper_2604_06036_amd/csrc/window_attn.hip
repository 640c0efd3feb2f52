// (d) Joint prefill attention of refresh + suffix tokens over the mixed window cache, gfx950.
//
// Paper Sec. 3.5: refresh tokens and the normal suffix run one joint prefill pass; at each layer
// causal attention reads a cache that mixes reused (position-corrected) states with states
// written in the current pass.  Causality follows the window-sequence index of each query.
//
// bf16 kernels (matrix cores).  A workgroup = 4 waves = a tile of 128 "rows", a row being one
// (query token, query head of one kv group) pair, so the K/V tiles a workgroup stages in LDS are
// shared by all query heads of the group.  Keys are swept in tiles of 64 through LDS:
//   S^T = K Q^T      v_mfma_f32_32x32x16_bf16, A = K fragment from LDS (ds_read_b128),
//                    B = Q^T fragment held in registers for the whole sweep;
//   online softmax   fp32, per-lane statistics: in the S^T layout a lane owns one query and 16
//                    of its 32 keys, the two half-waves exchange the running max once per tile;
//   O^T += V^T P^T   P^T is already in B-operand layout (no LDS round trip); the V^T fragment is
//                    fetched from the row-major V tile with the LDS transpose read
//                    (ds_read_b64_tr_b16), so V is never transposed in memory.
// Tiles that lie wholly above a wave's causal frontier are skipped by that wave; only tiles that
// straddle a frontier pay for masking.  Cache rows past the workgroup's frontier are never read
// (they may be unallocated): the lanes that would fetch them fetch the frontier row instead.
//
// head_dim 128: a planning kernel lists the work items of the launch and persistent workgroups
// stream K/V tiles from HBM straight into LDS (global_load_lds), across item boundaries; long key
// sweeps of small batches are split over several items and merged by a second kernel.
// head_dim 64: one workgroup per row tile, tiles staged through registers.
//
// fp32 kernel: plain SIMT, one wave per (query, head), keys strided over lanes, online softmax
// per lane and a final cross-lane merge.  It exists for fp32 caches (small validation shapes).
#include <math.h>

#include "common.h"


namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

struct AttnParams {
  const void* __restrict__ q;
  const void* __restrict__ k;
  const void* __restrict__ v;
  void* __restrict__ out;
  const int32_t* __restrict__ cu_q;
  const int32_t* __restrict__ q_pos;
  const int32_t* __restrict__ block_table;
  const int32_t* __restrict__ kv_len;
  int64_t stride_slot, stride_head;
  int32_t max_blocks, n_streams, n_q_heads, n_kv_heads, group;
  float scale, scale_log2e;
  int64_t n_q;
  // split-KV (max_splits > 1): a row tile whose key sweep is longer than chunk_tiles key tiles is
  // shared by several work items; their un-normalised partial results go to the workspace and a
  // second kernel merges them (merging in the last workgroup to finish was built twice and is far
  // slower here, also with write-through stores in place of an L2 write-back: single stream,
  // 919 keys, 42 against 23 us per call; 6,033 keys 133 against 117; 17,630 keys 310 against 290)
  int32_t chunk_tiles, max_splits, bm, span;
  const int32_t* ws_plan;   // plan header (list offsets per XCD, row-tile count, end item, first items)
  const int32_t* ws_items;  // item descriptors, 8 ints each, the 8 XCD lists back to back
  // refresh write fused into the launch (cs_refresh_prefill_attn): rows to write before attention
  const void* __restrict__ k_new;
  const void* __restrict__ v_new;
  const int32_t* __restrict__ new_slot;
  int64_t n_new;
  int32_t row_vecs, head_vecs;   // 16-byte vectors per new row / per head
  int32_t* ws_sync;      // counters of the fused launch's launch-wide barrier (see launch_barrier)
  int32_t* ws_status;    // its status word
  int32_t* ws_desc;      // [items][8]: q0, rows_total, r_tile, kvh, n_split
  float* ws_ml;          // [items][max_splits][bm][2]: running max (raw score units), row sum
  float* ws_o;           // [items][max_splits][bm][128]: un-normalised output rows
};

constexpr int kBM = 128;   // rows per workgroup (4 waves x 32)
constexpr int kBN = 64;    // keys per LDS tile
constexpr float kNegInf = -INFINITY;
constexpr int kMaxBlocksInLds = 8192;   // block-table row staged in LDS: windows up to 131072 tokens

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// Two fp32 -> packed bf16 (round to nearest even) in one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Running-max slack of the online softmax, in log2 units: the reference maximum of a row is only
// raised (and the accumulators rescaled) when the tile maximum exceeds it by more than this, so
// probabilities stay below 2^kMaxSlack and almost every tile skips the rescale.
constexpr float kMaxSlack = 8.0f;

template <int D>
__global__ __launch_bounds__(256, 2) void window_attn_bf16_kernel(AttnParams p) {
  constexpr int KP = D + 8;            // K tile pitch (elements): rows shift by 4 banks
  constexpr int VP = D + 32;           // V tile pitch: rows shift by 16 banks (transpose reads)
  constexpr int STEPS = D / 16;        // contraction steps of S^T
  constexpr int DB = D / 32;           // 32-wide blocks of the head dimension in O^T
  constexpr int CPR = D / 8;           // 16-byte chunks per cache row
  constexpr int RPP = 256 / CPR;       // rows staged per pass by the whole workgroup
  constexpr int RPW = 64 / CPR;        // rows staged per pass by one wave (inside one cache block)
  constexpr int PASSES = kBN / RPP;
  constexpr int BPT = kBN / CS_KV_BLOCK;   // cache blocks per key tile

  __shared__ __attribute__((aligned(16))) uint16_t sK[kBN * KP];
  __shared__ __attribute__((aligned(16))) uint16_t sV[kBN * VP];
  extern __shared__ int32_t s_bt[];    // this stream's block-table row (max_blocks entries)

  // ---- which (stream, row tile) is this workgroup?  longest tiles of a stream come first
  int x = blockIdx.x, s = 0, q0 = 0, rows_total = 0, n_row_tiles = 0;
  for (; s < p.n_streams; ++s) {
    q0 = p.cu_q[s];
    rows_total = (p.cu_q[s + 1] - q0) * p.group;
    n_row_tiles = (rows_total + kBM - 1) / kBM;
    if (x < n_row_tiles) break;
    x -= n_row_tiles;
  }
  if (s == p.n_streams) return;
  const int r_tile = (n_row_tiles - 1 - x) * kBM;
  const int kvh = blockIdx.y;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;

  // ---- this lane's row (query token, head) and causal frontier
  const int row = r_tile + wave * 32 + n;
  const bool valid = row < rows_total;
  const int row_c = valid ? row : rows_total - 1;
  const int tok = q0 + row_c / p.group;
  const int head = kvh * p.group + row_c % p.group;
  // a frontier never lies past the entries the stream's block-table row defines
  const int cap = min(p.kv_len[s], p.max_blocks * CS_KV_BLOCK) - 1;
  const int lim = valid ? min(p.q_pos[tok], cap) : -1;

  const int wg_last = min(r_tile + kBM, rows_total) - 1;
  const int wg_max = min(p.q_pos[q0 + wg_last / p.group], cap);
  const int w_first = r_tile + wave * 32;
  const bool wave_live = w_first < rows_total;
  const int w_last = min(w_first + 31, rows_total - 1);
  const int wave_min = wave_live ? min(p.q_pos[q0 + w_first / p.group], cap) : -1;
  const int wave_max = wave_live ? min(p.q_pos[q0 + w_last / p.group], cap) : -1;
  if (wg_max < 0) return;                 // the stream defines no cache entry: nothing to attend to
  const int n_key_tiles = wg_max / kBN + 1;
  const int last_blk = wg_max / CS_KV_BLOCK;

  // ---- Q^T fragments: lane = (query n, half h) holds d-slice [16*step + 8h, +8)
  const uint16_t* qrow = static_cast<const uint16_t*>(p.q) +
                         (static_cast<int64_t>(tok) * p.n_q_heads + head) * D;
  bf16x8 qf[STEPS];
#pragma unroll
  for (int st = 0; st < STEPS; ++st)
    qf[st] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const cs::u32x4*>(qrow + 16 * st + 8 * h));

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = kNegInf, l_run = 0.f;
  const float slack = kMaxSlack / p.scale_log2e;          // in raw score units

  // ---- staging of K/V tiles.  Thread -> row st_row + pass * RPP of the tile, chunk st_chunk.
  // A wave's rows of one pass lie inside one 16-token cache block, so the block id is
  // wave-uniform and the per-lane part of the address never changes.
  const int st_row = tid / CPR, st_chunk = tid % CPR;
  const int32_t* bt = p.block_table + static_cast<int64_t>(s) * p.max_blocks;
  const int64_t lane_off = static_cast<int64_t>(st_row % CS_KV_BLOCK) * p.stride_slot +
                           static_cast<int64_t>(kvh) * p.stride_head + st_chunk * 8;
  const uint16_t* kbase = static_cast<const uint16_t*>(p.k) + lane_off;
  const uint16_t* vbase = static_cast<const uint16_t*>(p.v) + lane_off;
  const int64_t blk_stride = static_cast<int64_t>(CS_KV_BLOCK) * p.stride_slot;
  cs::u32x4 kreg[PASSES], vreg[PASSES];

  for (int i = tid; i <= last_blk; i += 256) s_bt[i] = bt[i];
  __syncthreads();

  // Full tiles: every row is a live cache entry.  The last tile may end inside a block (rows past
  // the frontier are staged as zeros: they can hold anything) or before a block the table does
  // not define (never read).
  auto fetch = [&](int key_tile, bool last) {
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      const int bi = key_tile * BPT + (i * RPP + wave * RPW) / CS_KV_BLOCK;     // wave-uniform
      if (!last || bi <= last_blk) {
        const int64_t blk = __builtin_amdgcn_readfirstlane(s_bt[bi]);
        kreg[i] = *reinterpret_cast<const cs::u32x4*>(kbase + blk * blk_stride);
        vreg[i] = *reinterpret_cast<const cs::u32x4*>(vbase + blk * blk_stride);
      }
      if (last && (bi > last_blk || key_tile * kBN + st_row + i * RPP > wg_max)) {
        kreg[i] = cs::u32x4{0, 0, 0, 0};
        vreg[i] = cs::u32x4{0, 0, 0, 0};
      }
    }
  };

  if (n_key_tiles == 1) fetch(0, true); else fetch(0, false);
  for (int kt = 0; kt < n_key_tiles; ++kt) {
    __syncthreads();                       // everyone is done reading the previous tile
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      const int r = st_row + i * RPP;
      *reinterpret_cast<cs::u32x4*>(&sK[r * KP + st_chunk * 8]) = kreg[i];
      *reinterpret_cast<cs::u32x4*>(&sV[r * VP + st_chunk * 8]) = vreg[i];
    }
    __syncthreads();
    if (kt + 2 < n_key_tiles) fetch(kt + 1, false);
    else if (kt + 1 < n_key_tiles) fetch(kt + 1, true);

    const int j0 = kt * kBN;
    if (j0 > wave_max) continue;           // wholly above this wave's frontier (wave-uniform)

    // ---- S^T = K Q^T for the 64 keys of the tile: two 32-key blocks, MFMAs alternate between
    //      the two accumulators so that consecutive ones are independent
    f32x16 sacc[2];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8 a = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const cs::u32x4*>(&sK[(kb * 32 + n) * KP + 16 * st + 8 * h]));
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[st], st == 0 ? zero16 : sacc[kb], 0, 0, 0);
      }
    }
    // register r of block kb is key j0 + 32 kb + 8 (r / 4) + 4 h + r % 4 of query n
    if (j0 + kBN - 1 > wave_min) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + 32 * kb + 8 * (r / 4) + 4 * h + (r % 4);
          if (key > lim) sacc[kb][r] = kNegInf;
        }
    }
    float t_max = kNegInf;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) t_max = fmaxf(t_max, sacc[kb][r]);
    t_max = fmaxf(t_max, __shfl_xor(t_max, 32));
    // raise the row's reference maximum only when the tile exceeds it by more than the slack
    // (always on the first visible key: m_run = -inf); both half-waves take the same decision
    if (__any(t_max > m_run + slack)) {
      const bool up = t_max > m_run + slack;
      const float m_new = up ? t_max : m_run;
      const float alpha = up ? __builtin_amdgcn_exp2f((m_run - m_new) * p.scale_log2e) : 1.f;
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    }
    const float m_scaled = (m_run == kNegInf ? 0.f : m_run) * p.scale_log2e;

    // ---- P = exp2(S c - m c), packed to bf16 in B-operand order.  MFMA (kb, mm) contracts S
    //      registers 8mm..8mm+7 of block kb; slot 8h + i of the contraction is key
    //      32 kb + 16 mm + 8 (i / 4) + 4 h + i % 4.  Row sums are taken over the rounded values.
    bf16x8 pb[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        cs::u32x4 w;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float e0 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][8 * mm + 2 * c], p.scale_log2e, -m_scaled));
          const float e1 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][8 * mm + 2 * c + 1], p.scale_log2e, -m_scaled));
          const uint32_t pk = pack_bf16x2(e0, e1);
          l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk),
                                                  __builtin_bit_cast(bf16x2, 0x3f803f80u), l_run, false);
          w[c] = pk;
        }
        pb[kb][mm] = __builtin_bit_cast(bf16x8, w);
      }

    // ---- O^T += V^T P^T.  Transpose read: lane i of a 16-lane group supplies
    //      &V[key0 + i / 4][col0 + 4 (i % 4)] and receives V[key0 + 0..3][col0 + i]
    const int i16 = lane & 15, gid = (lane >> 4) & 1;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const int key0 = 32 * kb + 16 * mm + 4 * h + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const int col = 32 * db + 16 * gid + 4 * (i16 & 3);
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (lds_s16x4*)(&sV[key0 * VP + col]));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (lds_s16x4*)(&sV[(key0 + 8) * VP + col]));
          const s16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), pb[kb][mm],
                                                         o[db], 0, 0, 0);
        }
      }
  }

  // ---- normalise and store: register r of block db is d = 32 db + 8 (r / 4) + 4 h + r % 4
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (valid) {
    const float inv = 1.f / l_tot;
    uint16_t* orow = static_cast<uint16_t*>(p.out) +
                     (static_cast<int64_t>(tok) * p.n_q_heads + head) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        cs::u32x2 w;
        w.x = pack_bf16x2(o[db][4 * rq + 0] * inv, o[db][4 * rq + 1] * inv);
        w.y = pack_bf16x2(o[db][4 * rq + 2] * inv, o[db][4 * rq + 3] * inv);
        *reinterpret_cast<cs::u32x2*>(orow + 32 * db + 8 * rq + 4 * h) = w;
      }
  }
}

// ------------------------------------------------------------------------------------------
// Tile transport for head_dim 128 (the shape of every bf16 workload measured).
//
// K/V tiles are copied global -> LDS by the DMA form of the global load
// (global_load_lds_dwordx4: lane l of a wave deposits its 16 bytes at base + 16 l, the source
// address is free per lane), so nothing is staged through registers and there is one workgroup
// barrier per tile.  Because the DMA fixes the LDS position of each lane's chunk, bank conflicts
// are avoided by choosing WHICH 16-byte chunk of a row each lane fetches (an XOR swizzle on the
// source side) instead of padding rows:
//   K tile row r: chunk c is stored at position c ^ (r % 16)   (ds_read_b128 of 16 rows at one c)
//   V tile row r: chunk c is stored at position c ^ (4 (r % 4) + 2 ((r / 4) % 2))
//                 (a transpose read touches 8 rows x 2 chunks: this spreads them over all banks)
typedef __attribute__((address_space(3))) void lds_void_t;

// One 16-byte-per-lane DMA copy global -> LDS (lane l lands at lds_addr + 16 l).  Issued as inline
// assembly on purpose: the compiler then keeps no scoreboard entry for it and does not drain the
// whole prefetch queue before the next LDS read; completion is enforced by the explicit vmcnt
// waits and workgroup barriers of the pipeline below.  The "memory" clobber tells the compiler
// that LDS contents change here.
__device__ __forceinline__ void dma16(const void* gsrc, const void* lds_dst) {
  const uint32_t lds_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void_t*)lds_dst));
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(gsrc), "s"(lds_addr)
               : "memory", "m0");
}

// The same with a wave-uniform 64-bit base in SGPRs and a 32-bit byte offset per lane.
__device__ __forceinline__ void dma16_s(uint32_t off, const void* sbase, const void* lds_dst) {
  const uint32_t lds_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void_t*)lds_dst));
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(off), "s"(sbase), "s"(lds_addr)
               : "memory", "m0");
}

// ... and with the LDS destination given as a byte address in an SGPR.
__device__ __forceinline__ uint32_t lds_address(const void* lds_ptr) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void_t*)lds_ptr));
}
__device__ __forceinline__ void dma16_sa(uint32_t off, const void* sbase, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(off), "s"(sbase), "s"(lds_addr)
               : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  // s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in bits
  // 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8 left at their maxima)
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// =============================================================================================
// bf16 / head_dim 128: planned, persistent kernel
//
// A small planning kernel turns (cu_q, q_pos) into a list of work items, an item being one
// (stream, kv head, 128-row tile, key range), and deals the items to the 8 XCDs: all items of one
// (stream, kv head) pair go to one XCD (their K/V tiles then meet in that XCD's L2), pairs are
// dealt to XCDs in boustrophedon order of decreasing work, and every XCD's list is sorted by
// decreasing key-range length.  The plan depends only on cu_q and q_pos, so one plan serves
// every decoder layer of a step.
//
// The attention kernel is persistent: workgroup b serves XCD b % 8 (workgroups are dealt to XCDs
// round robin by the hardware) and takes the items at positions j, 2S-1-j, 2S+j, ... of that list
// (j = b / 8, S workgroups per XCD): with a sorted list this alternation evens out the totals
// without any run-time queue.  Its K/V tile requests run one tile ahead of the computation ACROSS
// item boundaries, item descriptors and cache-block ids arrive through scalar loads issued a tile
// ahead of their use, and the Q rows of the next item are requested before the finished item is
// normalised and stored, so that the per-item latencies (descriptor -> block table -> first tile)
// that dominate short key sweeps are paid once per workgroup instead of once per item.

typedef __attribute__((ext_vector_type(8))) int32_t i32x8;

// Item descriptor: 8 ints.  [0] first query token of the stream, [1] rows of the stream (tokens x
// heads per kv group), [2] first row of the tile, [3] kv head | stream << 8, [4] highest visible
// cache index among the tile's rows, [5] key tiles [begin, end) as begin | end << 16, [6] index of
// the item the same workgroup takes next (-1: none), [7] first row of the item's partial result in
// the workspace, or -1 when the item covers the whole sweep and writes `out`.
// Plan header (ints): [0..8] list offsets per XCD, [9] row tiles, [16..23] end item,
// then one 32-int entry per workgroup j of XCD x at [32 + 32 (64 x + j)]: [0..2] its first three
// items (-1: none), [3] cache block of its first item's frontier, [4..7] cache blocks of its first
// tile request (one per wave), [8..15] a copy of its first item's descriptor, [16] its item count.
// With the entry a workgroup can send its first tile request after ONE dependent load.
constexpr int kSlotsPerXcd = 64;      // persistent workgroups per XCD: 32 CUs x 2
constexpr int kHdrEndItem = 16, kHdrHeads = 32;
constexpr int kHdrEntryInts = 32;
constexpr int kHdrStatus = 14;        // status word of the fused launch's launch-wide wait
// Behind the entries, the counters of that wait, 256 bytes apart so that they sit in different
// memory channels: kSyncGroups group counters, the counter of finished groups, the release word.
constexpr int kSyncGroups = 16, kSyncPitch = 64;
constexpr int kHdrSyncBase = (kHdrHeads + kHdrEntryInts * 8 * kSlotsPerXcd + kSyncPitch - 1) / kSyncPitch * kSyncPitch;
constexpr int kSyncInts = (kSyncGroups + 2) * kSyncPitch;
constexpr int kPlanHeaderInts = kHdrSyncBase + kSyncInts;
constexpr int kItemFixedCostHalves = 3;  // per-item overhead in half key tiles, for the planner's balance
constexpr int kPlanThreads = 1024;
constexpr int kSortMax = 2048;        // streams sorted by work in LDS; beyond, stream order is kept

struct PlanParams {
  const int32_t* __restrict__ cu_q;
  const int32_t* __restrict__ q_pos;
  const int32_t* __restrict__ block_table;
  const int32_t* __restrict__ kv_len;
  int32_t max_blocks;
  int32_t n_streams, group, n_kv_heads, chunk_tiles, max_splits, max_tiles, r_cap, bm, n_slots, hist_pitch;   // n_slots: workgroups per XCD
  int32_t* header;      // [kPlanHeaderInts]
  int32_t* items;       // [items_cap][8]
  int32_t* rt_desc;     // [r_cap * n_kv_heads][8]: q0, rows_total, r_tile, kvh, n_split
  int32_t* st_toff;     // [n_streams + 1] first row tile of each stream
  int32_t* st_work;     // [n_streams] key tiles summed over the stream's row tiles
  int32_t* st_rank;     // [n_streams] rank by decreasing work
  int32_t* rt_stream;   // [r_cap]
  int32_t* rt_wgmax;    // [r_cap]
  int32_t* hist;        // [8][hist_pitch] items per (XCD, bucket), then list cursors
  int32_t span;         // 1: sweeps are cut into contiguous spans of equal cost (few, long sweeps)
  int32_t pref_pitch;   // ints per XCD in sw_pref
  int32_t* sw_pref;     // [8][pref_pitch] span plan: cost prefix of each XCD's sweeps
};

// Exclusive prefix sum over the kPlanThreads threads of the planning workgroup.
__device__ __forceinline__ int plan_block_scan(int v, int* s_wave, int& total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_up(incl, off);
    if (lane >= off) incl += t;
  }
  __syncthreads();                       // s_wave may still be read from a previous call
  if (lane == 63) s_wave[w] = incl;
  __syncthreads();
  int base = 0, sum = 0;
  for (int i = 0; i < kPlanThreads / 64; ++i) {
    const int t = s_wave[i];
    if (i < w) base += t;
    sum += t;
  }
  total = sum;
  return base + incl - v;
}

// Rows (query tokens x query heads of one kv group) of a stream; a stream whose block-table row
// defines no entry (kv_len <= 0) has nothing to attend to and gets no row tiles.
__device__ __forceinline__ int plan_stream_rows(const PlanParams& pp, int s) {
  return pp.kv_len[s] > 0 ? (pp.cu_q[s + 1] - pp.cu_q[s]) * pp.group : 0;
}

__device__ __forceinline__ int plan_xcd_of_pair(int pair) {
  const int round = pair >> 3, pos = pair & 7;
  return (round & 1) ? 7 - pos : pos;
}

// Span plan, for launches with few (row tile, kv head) sweeps, some of them long (one stream with
// a long window; any small batch).  Dealing whole sweeps, or fixed key ranges of them, to workgroups
// leaves the workgroups with unequal totals because the pieces are coarse next to a workgroup's
// share.  Here every XCD gets every eighth sweep (sweep = row tile * kv heads + kv head, so with
// four or eight kv heads an XCD serves one kv head), lays its sweeps end to end, and the sequence
// is cut into one contiguous span per workgroup, of equal COST: 2 n_kt + kItemFixedCostHalves per
// sweep, in half key tiles, the second workgroup of a CU (slots 32..63) getting 3/4 of the first
// one's share because the issue arbiter serves it less often.  A sweep that a cut crosses becomes
// several items whose partial results the merge kernel combines; cuts closer than kMinPieceTiles to
// a sweep's end move onto it.  Items of a workgroup are consecutive in the list, pieces of a sweep
// are consecutive too, and the position of an item in the list also names its partial-result slot.
constexpr int kMinSpanTiles = 3;     // fewer workgroups are used rather than give one less than this
constexpr int kMinPieceTiles = 2;
constexpr int kSpanWeightFirst = 4, kSpanWeightSecond = 3;

constexpr int kSpanPrefInLds = 8 * 136;   // the span plan runs with fewer than 1,024 sweeps: at most 130 ints per XCD

__device__ void plan_spans(const PlanParams& pp, int n_rt, int* s_wave, int (*s_cut)[kSlotsPerXcd + 1], int* s_pref) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n_kv = pp.n_kv_heads;
  const int n_sw = n_rt * n_kv;
  auto sweep_tiles = [&](int sw) { return max(pp.rt_wgmax[sw / n_kv], 0) / kBN + 1; };
  // ---- cost prefix of every XCD's sweeps (one wave per XCD)
  if (w < 8) {
    int32_t* pref = pp.sw_pref + w * pp.pref_pitch;
    const int n_x = (n_sw - w + 7) >> 3;
    int run = 0;
    if (lane == 0) pref[0] = 0;
    for (int i0 = 0; i0 < n_x; i0 += 64) {
      const int i = i0 + lane;
      const int v = i < n_x ? 2 * sweep_tiles(8 * i + w) + kItemFixedCostHalves : 0;
      int incl = v;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
      }
      if (i < n_x) pref[i + 1] = run + incl;
      run += __shfl(incl, 63);
    }
  }
  __threadfence_block();
  __syncthreads();
  // the searches below read the prefixes many times: keep them in LDS when they fit (they do for
  // every launch the host routes here; the global copy serves the general case)
  const bool in_lds = 8 * pp.pref_pitch <= kSpanPrefInLds;
  if (in_lds)
    for (int i = tid; i < 8 * pp.pref_pitch; i += kPlanThreads)
      s_pref[i] = __hip_atomic_load(&pp.sw_pref[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  // Position helpers of XCD x.  A position is a tile count from the start of the XCD's sequence.
  auto n_of = [&](int x) { return (n_sw - x + 7) >> 3; };
  auto cost_pref = [&](int x, int i) {
    return in_lds ? s_pref[x * pp.pref_pitch + i]
                  : __hip_atomic_load(&pp.sw_pref[x * pp.pref_pitch + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
  auto tile_pref = [&](int x, int i) { return (cost_pref(x, i) - kItemFixedCostHalves * i) >> 1; };
  auto sweep_at_tile = [&](int x, int pos) {      // largest i with tile_pref(i) <= pos (pos < total tiles)
    int lo = 0, hi = n_of(x);
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (tile_pref(x, mid) <= pos) lo = mid; else hi = mid;
    }
    return lo;
  };
  // ---- cuts: thread (x, j) places the start of workgroup j's span
  const int x = tid >> 6, j = tid & 63;          // threads 0..511: one per (XCD, workgroup)
  const int n_wg = min(pp.n_slots, kSlotsPerXcd);
  if (tid < 512) {
    const int n_x = n_of(x);
    const int total_tiles = n_x > 0 ? tile_pref(x, n_x) : 0;
    const int total_cost = n_x > 0 ? cost_pref(x, n_x) : 0;
    const int spans = total_tiles > 0 ? max(1, min(n_wg, total_tiles / kMinSpanTiles)) : 0;
    auto weight_before = [&](int k) { return k <= 32 ? kSpanWeightFirst * k : kSpanWeightFirst * 32 + kSpanWeightSecond * (k - 32); };
    int cut = total_tiles;
    if (j < spans) {
      const int64_t c = static_cast<int64_t>(total_cost) * weight_before(j) / weight_before(spans);   // cost position
      int lo = 0, hi = n_x;                       // largest i with cost_pref(i) <= c
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cost_pref(x, mid) <= c) lo = mid; else hi = mid;
      }
      const int len = sweep_tiles(8 * lo + x);
      int o = static_cast<int>(c - cost_pref(x, lo) - kItemFixedCostHalves + 1) >> 1;
      o = max(0, min(o, len));
      if (o < kMinPieceTiles) o = 0;
      if (len - o < kMinPieceTiles) o = len;
      cut = j == 0 ? 0 : tile_pref(x, lo) + o;
    }
    s_cut[x][j] = cut;
    if (j == 0) s_cut[x][kSlotsPerXcd] = total_tiles;
  }
  __syncthreads();
  // ---- items per workgroup, their positions in the list
  int i_lo = 0, i_hi = -1, lo_t = 0, hi_t = 0;
  if (tid < 512) {
    lo_t = s_cut[x][j];
    hi_t = s_cut[x][j + 1];
    if (hi_t > lo_t) {
      i_lo = sweep_at_tile(x, lo_t);
      i_hi = sweep_at_tile(x, hi_t - 1);
    }
  }
  const int count = i_hi - i_lo + 1;
  int total_items;
  const int first = plan_block_scan(tid < 512 ? count : 0, s_wave, total_items);
  if (tid < 512 && j == 0) pp.header[x] = first;
  if (tid == 0) {
    pp.header[8] = total_items;
    pp.header[9] = n_sw;
    for (int i = 10; i < kHdrHeads; ++i) pp.header[i] = 0;
    pp.header[kHdrEndItem + 4] = -1;                    // end item: no key tiles, nothing visible
    pp.header[kHdrEndItem + 6] = -1;
    pp.header[kHdrEndItem + 7] = -1;
  }
  for (int i = tid; i < kSyncInts; i += kPlanThreads) pp.header[kHdrSyncBase + i] = 0;
  for (int i = n_sw + tid; i < pp.r_cap * n_kv; i += kPlanThreads)
    pp.rt_desc[static_cast<int64_t>(i) * 8 + 4] = 0;
  if (tid >= 512) return;
  // ---- write the items of workgroup (x, j) and its header entry
  int32_t d_first[8] = {0, 0, 0, 0, -1, 0, -1, -1};     // the end item
  for (int i = i_lo; i <= i_hi; ++i) {
    const int sw = 8 * i + x;
    const int r = sw / n_kv, kvh = sw - r * n_kv;
    const int s = pp.rt_stream[r];
    const int t = r - pp.st_toff[s];
    const int q0 = pp.cu_q[s];
    const int rows = plan_stream_rows(pp, s);
    const int wg_max = pp.rt_wgmax[r];
    const int begin = tile_pref(x, i), n_kt = tile_pref(x, i + 1) - begin;
    const int kb = max(lo_t, begin) - begin, ke = min(hi_t, begin + n_kt) - begin;
    const int pos = first + (i - i_lo);
    const bool split = kb > 0 || ke < n_kt;
    int32_t d[8] = {q0, rows, t * pp.bm, kvh | (s << 8), wg_max, kb | (ke << 16), i < i_hi ? pos + 1 : -1,
                    split ? pos * pp.bm : -1};
    int32_t* it = pp.items + static_cast<int64_t>(pos) * 8;
#pragma unroll
    for (int k = 0; k < 8; ++k) it[k] = d[k];
    if (i == i_lo) {
#pragma unroll
      for (int k = 0; k < 8; ++k) d_first[k] = d[k];
    }
    if (kb == 0) {                                       // the sweep's first piece describes it to the merge kernel
      int pieces = 1;
      for (int k = 1; k < kSlotsPerXcd; ++k) {
        const int c = s_cut[x][k];
        pieces += (c > begin && c < begin + n_kt && c != s_cut[x][k - 1]) ? 1 : 0;
      }
      int32_t* rd = pp.rt_desc + static_cast<int64_t>(sw) * 8;
      rd[0] = q0; rd[1] = rows; rd[2] = t * pp.bm; rd[3] = kvh; rd[4] = pieces; rd[5] = pos;
    }
  }
  int32_t* hd = pp.header + kHdrHeads + kHdrEntryInts * (x * kSlotsPerXcd + j);
  int32_t ids[4] = {0, 0, 0, 0}, last_id = 0;
  if (count > 0) {
    const int32_t* row = pp.block_table + static_cast<int64_t>(d_first[3] >> 8) * pp.max_blocks;
    const int last_blk = max(d_first[4], 0) >> 4;
    for (int i = 0; i < 4; ++i) ids[i] = row[min((d_first[5] & 0xffff) * 4 + i, last_blk)];
    last_id = row[last_blk];
  }
  hd[0] = count > 0 ? first : -1; hd[1] = count > 1 ? first + 1 : -1; hd[2] = count > 2 ? first + 2 : -1; hd[3] = last_id;
  for (int i = 0; i < 4; ++i) hd[4 + i] = ids[i];
  for (int i = 0; i < 8; ++i) hd[8 + i] = d_first[i];
  hd[16] = count;
}

__global__ __launch_bounds__(kPlanThreads) void window_attn_plan_kernel(PlanParams pp) {
  __shared__ int s_wave[kPlanThreads / 64];
  __shared__ unsigned long long s_key[kSortMax];
  __shared__ int s_list_off[9];
  __shared__ int s_by_rank[8][64];      // deal: lane (and length) of the item of each rank, per XCD
  __shared__ int s_cut[8][kSlotsPerXcd + 1];   // span plan: first tile position of every workgroup's span
  const int tid = threadIdx.x;
  const int hist_pitch = pp.hist_pitch;

  // ---- clear counters; row tiles per stream
  for (int i = tid; i < 8 * hist_pitch; i += kPlanThreads) pp.hist[i] = 0;
  int carry = 0;
  for (int s0 = 0; s0 < pp.n_streams; s0 += kPlanThreads) {
    const int s = s0 + tid;
    int tiles = 0;
    if (s < pp.n_streams) {
      const int rows = plan_stream_rows(pp, s);
      tiles = (rows + pp.bm - 1) / pp.bm;
      pp.st_work[s] = 0;
    }
    int total;
    const int excl = plan_block_scan(tiles, s_wave, total);
    if (s < pp.n_streams) pp.st_toff[s] = carry + excl;
    carry += total;
  }
  const int n_rt = carry;                // row tiles per kv head
  if (tid == 0) pp.st_toff[pp.n_streams] = n_rt;
  __threadfence_block();
  __syncthreads();

  // ---- per row tile: its stream, its causal frontier; work per stream
  for (int r = tid; r < n_rt; r += kPlanThreads) {
    int lo = 0, hi = pp.n_streams;       // last stream whose first row tile is <= r
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (pp.st_toff[mid] <= r) lo = mid; else hi = mid;
    }
    const int s = lo;
    const int t = r - pp.st_toff[s];
    const int q0 = pp.cu_q[s];
    const int rows = plan_stream_rows(pp, s);
    const int last_row = min((t + 1) * pp.bm, rows) - 1;
    // the tile's frontier, kept inside the entries the stream's block-table row defines
    const int wg_max = max(0, min(pp.q_pos[q0 + last_row / pp.group], min(pp.kv_len[s], pp.max_blocks * CS_KV_BLOCK) - 1));
    pp.rt_stream[r] = s;
    pp.rt_wgmax[r] = wg_max;
    atomicAdd(&pp.st_work[s], max(wg_max, 0) / kBN + 1);
  }
  __threadfence_block();
  __syncthreads();

  if (pp.span) {
    plan_spans(pp, n_rt, s_wave, s_cut, reinterpret_cast<int*>(s_key));    // s_key is unused on this route
    return;
  }

  // ---- rank streams by decreasing work (ties: stream order)
  if (pp.n_streams <= kSortMax) {
    int n_sort = 1;
    while (n_sort < pp.n_streams) n_sort <<= 1;
    for (int i = tid; i < n_sort; i += kPlanThreads)
      s_key[i] = i < pp.n_streams
                     ? (static_cast<unsigned long long>(0x7fffffff - __hip_atomic_load(&pp.st_work[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) << 32) | static_cast<unsigned>(i)
                     : ~0ull;
    __syncthreads();
    for (int k = 2; k <= n_sort; k <<= 1)
      for (int j = k >> 1; j > 0; j >>= 1) {
        for (int i = tid; i < n_sort; i += kPlanThreads) {
          const int partner = i ^ j;
          if (partner > i) {
            const unsigned long long a = s_key[i], b = s_key[partner];
            const bool up = (i & k) == 0;
            if ((a > b) == up) { s_key[i] = b; s_key[partner] = a; }
          }
        }
        __syncthreads();
      }
    for (int i = tid; i < pp.n_streams; i += kPlanThreads)
      pp.st_rank[static_cast<unsigned>(s_key[i] & 0xffffffffu)] = i;
  } else {
    for (int i = tid; i < pp.n_streams; i += kPlanThreads) pp.st_rank[i] = i;
  }
  __threadfence_block();
  __syncthreads();

  // ---- order of an XCD's list.  With enough (stream, kv head) pairs to give every XCD two, a pair
  //      goes to one XCD whole (boustrophedon deal by rank) and its row tiles stay together in the
  //      list, pairs by rank, longest row tile first: the workgroups of an XCD then sweep the K/V
  //      of few pairs at a time and share them in its L2 (an order by length alone re-read K/V
  //      2.5 times from HBM).  Otherwise items are dealt round robin and ordered by length.
  //      bucket = position class in the list (counting sort), XCD chosen alongside.
  const bool grouped = pp.n_streams * pp.n_kv_heads >= 16;
  auto place = [&](int r, int s, int kvh, int split, int len, int& bucket) {
    if (grouped) {
      const int pair = pp.st_rank[s] * pp.n_kv_heads + kvh;
      bucket = pair >> 3;
      return plan_xcd_of_pair(pair);
    }
    bucket = pp.max_tiles + 1 - min(len, pp.max_tiles + 1);
    return (r * pp.n_kv_heads + kvh + split) & 7;
  };
  for (int r = tid; r < n_rt; r += kPlanThreads) {
    const int s = pp.rt_stream[r];
    const int n_kt = max(pp.rt_wgmax[r], 0) / kBN + 1;
    const int n_split = pp.max_splits > 1 ? min((n_kt + pp.chunk_tiles - 1) / pp.chunk_tiles, pp.max_splits) : 1;
    for (int kvh = 0; kvh < pp.n_kv_heads; ++kvh)
      for (int c = 0; c < n_split; ++c) {
        const int len = n_split > 1 ? min(pp.chunk_tiles, n_kt - c * pp.chunk_tiles) : n_kt;
        int bucket;
        const int x = place(r, s, kvh, c, len, bucket);
        atomicAdd(&pp.hist[x * hist_pitch + bucket], 1);
      }
  }
  __threadfence_block();
  __syncthreads();

  // ---- per XCD (one wave each): first list position of every bucket
  {
    const int w = tid >> 6, lane = tid & 63;
    if (w < 8) {
      int* hx = pp.hist + w * hist_pitch;
      int run = 0;
      for (int k0 = 0; k0 < hist_pitch; k0 += 64) {
        const int k = k0 + lane;
        const int v = k < hist_pitch ? __hip_atomic_load(&hx[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
        int incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const int t = __shfl_up(incl, off);
          if (lane >= off) incl += t;
        }
        if (k < hist_pitch) hx[k] = run + incl - v;
        run += __shfl(incl, 63);
      }
      if (lane == 0) s_list_off[w + 1] = run;          // list length for now
    }
  }
  __syncthreads();
  if (tid == 0) {
    s_list_off[0] = 0;
    for (int x = 0; x < 8; ++x) s_list_off[x + 1] += s_list_off[x];
    for (int x = 0; x < 9; ++x) pp.header[x] = s_list_off[x];
    pp.header[9] = n_rt * pp.n_kv_heads;
    for (int i = 10; i < kHdrHeads; ++i) pp.header[i] = 0;
    pp.header[kHdrEndItem + 4] = -1;                    // end item: no key tiles, nothing visible
    pp.header[kHdrEndItem + 6] = -1;
    pp.header[kHdrEndItem + 7] = -1;
  }
  for (int i = tid; i < kSyncInts; i += kPlanThreads) pp.header[kHdrSyncBase + i] = 0;
  __threadfence_block();
  __syncthreads();

  // ---- write the items (row-tile slots beyond the planned ones are marked unsplit, so that the
  //      merge kernel needs no other bound than the size of its grid)
  for (int i = n_rt * pp.n_kv_heads + tid; i < pp.r_cap * pp.n_kv_heads; i += kPlanThreads)
    pp.rt_desc[static_cast<int64_t>(i) * 8 + 4] = 0;
  for (int r = tid; r < n_rt; r += kPlanThreads) {
    const int s = pp.rt_stream[r];
    const int t = r - pp.st_toff[s];
    const int q0 = pp.cu_q[s];
    const int rows = plan_stream_rows(pp, s);
    const int tiles_s = (rows + pp.bm - 1) / pp.bm;
    const int wg_max = pp.rt_wgmax[r];
    const int n_kt = max(wg_max, 0) / kBN + 1;
    const int n_split = pp.max_splits > 1 ? min((n_kt + pp.chunk_tiles - 1) / pp.chunk_tiles, pp.max_splits) : 1;
    for (int kvh = 0; kvh < pp.n_kv_heads; ++kvh) {
      const int rt_id = r * pp.n_kv_heads + kvh;
      int32_t* rd = pp.rt_desc + static_cast<int64_t>(rt_id) * 8;
      rd[0] = q0; rd[1] = rows; rd[2] = t * pp.bm; rd[3] = kvh; rd[4] = n_split;
      for (int c = 0; c < n_split; ++c) {
        const int kb = n_split > 1 ? c * pp.chunk_tiles : 0;
        const int ke = n_split > 1 ? min(n_kt, kb + pp.chunk_tiles) : n_kt;
        int bucket;
        const int x = place(r, s, kvh, c, ke - kb, bucket);
        int* cursor = &pp.hist[x * hist_pitch + bucket];
        // a pair's bucket holds its row tiles only: the longest (last) row tile goes first; where
        // sweeps are split or buckets are shared, arrival order decides
        const int within = grouped && pp.max_splits == 1 ? tiles_s - 1 - t : atomicAdd(cursor, 1);
        const int start = grouped && pp.max_splits == 1 ? __hip_atomic_load(cursor, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
        const int pos = s_list_off[x] + start + within;
        int32_t* it = pp.items + static_cast<int64_t>(pos) * 8;
        it[0] = q0; it[1] = rows; it[2] = t * pp.bm; it[3] = kvh | (s << 8); it[4] = wg_max;
        it[5] = kb | (ke << 16); it[6] = -1;
        it[7] = n_split > 1 ? (rt_id * pp.max_splits + c) * pp.bm : -1;
      }
    }
  }
  __threadfence_block();
  __syncthreads();

  // ---- deal every XCD's list to its workgroups (one wave per XCD, a lane per workgroup), a batch
  //      of as many items as there are workgroups at a time: within a batch the longest item goes
  //      to the workgroup with the least work so far, the second longest to the next one, ...
  //      (ranks by counting, 64 lane reads each).  This is close to the schedule a run-time queue
  //      would produce, fixed here so that the attention kernel needs no atomics.  Items of one
  //      workgroup are chained through their `next` field.
  {
    const int w = tid >> 6, lane = tid & 63;
    if (w < 8) {
      const int begin = s_list_off[w], end = s_list_off[w + 1];
      const int n_wg = min(pp.n_slots, 64);
      int load = lane < n_wg ? 0 : 0x7fffffff;          // half key tiles; lanes beyond the grid rank last
      int last = -1, first3[3] = {-1, -1, -1}, taken = 0;
      // (a pair-ordered list that is not a whole number of batches starts with the short batch:
      // the full batches that follow even the loads out again, which a short batch at the end
      // cannot.  A list ordered by length keeps its batches aligned instead: workgroups that start
      // equal-length items together sweep the same key ranges together and share them in L2,
      // which is worth more there: 6 % on the dense long-window case.)
      int n_batch = grouped ? (end - begin) % n_wg : 0;
      if (n_batch == 0) n_batch = n_wg;
      for (int base = begin; base < end; base += n_batch, n_batch = n_wg) {
        const int n_here = min(n_batch, end - base);      // the last batch of a length-ordered list may be short
        int len = -1;                                     // lanes without an item rank last
        if (lane < n_here) {
          const int kbe = __hip_atomic_load(&pp.items[static_cast<int64_t>(base + lane) * 8 + 5], __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);
          len = (kbe >> 16) - (kbe & 0xffff);
        }
        int item_rank = 0, load_rank = 0;                 // by decreasing length / increasing load, ties by lane
#pragma unroll 8
        for (int j = 0; j < 64; ++j) {
          const int lj = __builtin_amdgcn_readlane(len, j), wj = __builtin_amdgcn_readlane(load, j);
          item_rank += (lj > len || (lj == len && j < lane)) ? 1 : 0;
          load_rank += (wj < load || (wj == load && j < lane)) ? 1 : 0;
        }
        s_by_rank[w][item_rank] = lane | (len << 8);
        __builtin_amdgcn_wave_barrier();
        if (load_rank < n_here) {
          const int got = s_by_rank[w][load_rank];
          const int idx = base + (got & 255);
          if (last >= 0) pp.items[static_cast<int64_t>(last) * 8 + 6] = idx;
          if (taken == 0) first3[0] = idx;
          if (taken == 1) first3[1] = idx;
          if (taken == 2) first3[2] = idx;
          ++taken;
          last = idx;
          load += (2 * (got >> 8) + kItemFixedCostHalves) * (lane >= 32 ? kSpanWeightFirst : kSpanWeightSecond);
        }
        __builtin_amdgcn_wave_barrier();
      }
      if (lane < kSlotsPerXcd) {
        int32_t* hd = pp.header + kHdrHeads + kHdrEntryInts * (w * kSlotsPerXcd + lane);
        int32_t d[8] = {0, 0, 0, 0, -1, 0, -1, -1};       // the end item
        int32_t ids[4] = {0, 0, 0, 0}, last_id = 0;
        if (taken > 0) {
          for (int i = 0; i < 8; ++i)
            d[i] = __hip_atomic_load(&pp.items[static_cast<int64_t>(first3[0]) * 8 + i], __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
          const int32_t* row = pp.block_table + static_cast<int64_t>(d[3] >> 8) * pp.max_blocks;
          const int last_blk = d[4] >> 4;
          for (int i = 0; i < 4; ++i) ids[i] = row[min((d[5] & 0xffff) * 4 + i, last_blk)];
          last_id = row[last_blk];
        }
        hd[0] = first3[0]; hd[1] = first3[1]; hd[2] = first3[2]; hd[3] = last_id;
        for (int i = 0; i < 4; ++i) hd[4 + i] = ids[i];
        for (int i = 0; i < 8; ++i) hd[8 + i] = d[i];
        hd[16] = taken;
      }
    }
  }
}


// Scalar loads issued by hand: the results are uniform, travel outside the vector-memory queue
// (so waiting for them never drains tile requests) and are only read after the explicit wait.
__device__ __forceinline__ i32x8 sload8(const void* ptr) {
  i32x8 v;
  asm volatile("s_load_dwordx8 %0, %1, 0x0" : "=&s"(v) : "s"(ptr));
  return v;
}
__device__ __forceinline__ int32_t sload1(const void* ptr) {
  int32_t v;
  asm volatile("s_load_dword %0, %1, 0x0" : "=&s"(v) : "s"(ptr));
  return v;
}

// RB = 32-row blocks per wave.  RB = 1 is what runs: 128-row items, two workgroups per CU (two
// waves per SIMD hide each other's latencies).  RB = 2 (256-row items, one workgroup per CU with
// the whole register file, every K and V fragment read from LDS feeding two MFMAs) passes the same
// tests but measured 15-25 % slower as it stands: with one wave per SIMD nothing hides the softmax
// arithmetic unless the loop is software-pipelined by hand, and half the scores land in AGPRs.
// 16-byte store that is written through the XCD's L2 to memory (agent scope), the cache policy an
// agent-scope atomic store carries: its acknowledgement (vmcnt) comes when the other XCDs can read
// the bytes, so a wait on vmcnt stands in for an L2 write-back.  The s_nop belongs to the store: a
// store of more than 8 bytes reads its data registers for a cycle after it issues, the compiler
// does not know that this statement is such a store, and it is free to reuse the data registers in
// the very next instruction (seen in an experiment: the next row's address landed in the first
// 8 bytes of a stored row).
__device__ __forceinline__ void store_agent(void* dst, const cs::u32x4& v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" :: "v"(dst), "v"(v) : "memory");
}
// Waits for the acknowledgements of this wave's stores.  Spelled out: the compiler does not know of
// stores issued from inline assembly, so a fence of its own may come without the wait.
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

constexpr uint32_t kBarrierSpinLimit = 1u << 24;

// Launch-wide barrier of a grid whose workgroups are all resident (at most 2 per CU on 256 CUs, by
// construction of the persistent grid).  Arrivals are counted in two levels so that no counter takes
// more than n/16 + 16 read-modify-writes in a row (they execute at the memory side, one after the
// other per address): workgroup b adds to group counter b & 15; whoever completes a group resets it
// and adds to the counter of finished groups; whoever completes that resets it and bumps the release
// word.  Everybody else polls the release word against the value it read before arriving (it cannot
// have moved yet: a bump needs every arrival, the reader's included).  Which workgroup runs where
// plays no part in the counting.  The wait is bounded: after kBarrierSpinLimit polls the workgroup
// raises the status word and goes on, so every wave exits even if part of the grid never became
// resident; the results of such a launch are not valid and the status word says so.
//
// Visibility across the XCDs' L2s: the rows written before the barrier are stored write-through at
// agent scope (see store_agent) and every wave waits for its stores' acknowledgements, so no L2
// write-back is needed on arrival (one per workgroup measured 16 us per launch, one per wave 40 us);
// after the release one thread per workgroup invalidates the CU's vector cache and the XCD's L2
// (they are shared by the workgroup's waves), which costs nothing measurable.
__device__ __forceinline__ void launch_barrier(int32_t* sync, int32_t* status, int n_workgroups) {
  wait_stores();                                           // the row stores are acknowledged
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (threadIdx.x == 0) {
    int32_t* group = sync + (blockIdx.x % kSyncGroups) * kSyncPitch;
    int32_t* groups_done = sync + kSyncGroups * kSyncPitch;
    int32_t* release = sync + (kSyncGroups + 1) * kSyncPitch;
    const int in_group = (n_workgroups - static_cast<int>(blockIdx.x % kSyncGroups) + kSyncGroups - 1) / kSyncGroups;
    const int n_groups = n_workgroups < kSyncGroups ? n_workgroups : kSyncGroups;
    const int r0 = __hip_atomic_load(release, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    bool last = false;
    if (__hip_atomic_fetch_add(group, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == in_group - 1) {
      __hip_atomic_store(group, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (__hip_atomic_fetch_add(groups_done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_groups - 1) {
        __hip_atomic_store(groups_done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(release, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last = true;
      }
    }
    if (!last) {
      uint32_t polls = 0;
      while (__hip_atomic_load(release, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == r0) {
        if (++polls > kBarrierSpinLimit) {                // never taken when the whole grid is resident
          __hip_atomic_store(status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
        __builtin_amdgcn_s_sleep(8);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

template <int RB, bool FUSE>
__global__ __launch_bounds__(256, RB == 1 ? 2 : 1) void window_attn_bf16_stream_kernel(AttnParams p) {
  constexpr int WROWS = 32 * RB;        // rows per wave
  constexpr int D = 128;
  constexpr int STEPS = D / 16, DB = D / 32;
  constexpr int TILE = kBN * D;         // elements of one K (or V) tile: 16 KiB, unpadded
  constexpr int IPW = 4;                // 1-KiB DMA instructions per wave, per tile, per tensor

  __shared__ __attribute__((aligned(1024))) uint16_t sK[2][TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t sV[2][TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t s_sink[4][512];   // see request_part

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;

  if constexpr (FUSE) {
    // ---- refresh write (Sec. 3.5: the K/V just computed go into the destination cache before
    //      attention reads it): the whole grid moves the new rows, 16 bytes of K and of V per
    //      thread and turn, then meets at a launch-wide barrier
    const int64_t n_units = p.n_new * p.row_vecs;
    const cs::u32x4* kn = static_cast<const cs::u32x4*>(p.k_new);
    const cs::u32x4* vn = static_cast<const cs::u32x4*>(p.v_new);
    uint16_t* kc = const_cast<uint16_t*>(static_cast<const uint16_t*>(p.k));
    uint16_t* vc = const_cast<uint16_t*>(static_cast<const uint16_t*>(p.v));
    for (int64_t unit = static_cast<int64_t>(blockIdx.x) * 256 + tid; unit < n_units;
         unit += static_cast<int64_t>(gridDim.x) * 256) {
      const int64_t tok = unit / p.row_vecs;
      const int rem = static_cast<int>(unit - tok * p.row_vecs);
      const int sl = p.new_slot[tok];
      if (sl < 0) continue;
      const int head = rem / p.head_vecs, c = rem - head * p.head_vecs;
      const int64_t dst = static_cast<int64_t>(sl) * p.stride_slot + head * p.stride_head + c * 8;
      const cs::u32x4 kv = __builtin_nontemporal_load(kn + unit);
      const cs::u32x4 vv = __builtin_nontemporal_load(vn + unit);
      store_agent(kc + dst, kv);
      store_agent(vc + dst, vv);
    }
    launch_barrier(p.ws_sync, p.ws_status, static_cast<int>(gridDim.x));
  }

  // ---- this workgroup's items: a chain through the `next` field of the descriptors, dealt by the
  //      planning kernel; three descriptors of look-ahead are kept loaded
  const int xcd = blockIdx.x & 7, slot_j = blockIdx.x >> 3;
  auto item_at = [&](int idx) -> const int32_t* {
    return idx >= 0 ? p.ws_items + static_cast<int64_t>(idx) * 8 : p.ws_plan + kHdrEndItem;
  };
  const int32_t* entry = p.ws_plan + kHdrHeads + kHdrEntryInts * (xcd * kSlotsPerXcd + slot_j);
  i32x8 e0 = sload8(entry), d0 = sload8(entry + 8);
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(e0), "+s"(d0));
  if ((d0[5] >> 16) == 0) return;       // nothing for this workgroup
  i32x8 d1 = sload8(item_at(e0[1])), d2 = sload8(item_at(e0[2]));   // waited for after the first tile request
  int seq0 = 0;                         // d0 is the seq0-th item of this workgroup

  // ---- constants of the lane: DMA sources inside a cache block, LDS read addresses
  const uint16_t* kall = static_cast<const uint16_t*>(p.k);
  const uint16_t* vall = static_cast<const uint16_t*>(p.v);
  const int64_t blk_stride = static_cast<int64_t>(CS_KV_BLOCK) * p.stride_slot;
  const int l_row = lane >> 4, l_pos = lane & 15;
  uint32_t k_off[IPW], v_off[IPW];      // byte offsets inside a cache block (the host checks the range)
  int k_chunk[IPW], v_chunk[IPW];
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int trow = 4 * (wave * IPW + i) + l_row;          // row of the tile, 0..63
    k_chunk[i] = l_pos ^ (trow & 15);
    v_chunk[i] = l_pos ^ (4 * (trow & 3) + 2 * ((trow >> 2) & 1));
    k_off[i] = static_cast<uint32_t>(((trow & 15) * p.stride_slot + k_chunk[i] * 8) * 2);
    v_off[i] = static_cast<uint32_t>(((trow & 15) * p.stride_slot + v_chunk[i] * 8) * 2);
  }
  int k_rd[STEPS];
#pragma unroll
  for (int st = 0; st < STEPS; ++st) k_rd[st] = n * D + (((2 * st + h) ^ (n & 15)) << 3);
  const int i16 = lane & 15, gid = (lane >> 4) & 1;
  const int v_row = 4 * h + (i16 >> 2);
  const int v_swz = 4 * (v_row & 3) + 2 * (v_row >> 2);
  int v_rd[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
    v_rd[db] = v_row * D + (((4 * db + 2 * gid + ((i16 & 3) >> 1)) ^ v_swz) << 3) + 4 * (i16 & 1);

  uint32_t k_addr[STEPS], v_addr[DB];   // LDS byte addresses of this lane's fragments in stage 0
#pragma unroll
  for (int st = 0; st < STEPS; ++st) k_addr[st] = lds_address(&sK[0][0]) + 2 * k_rd[st];
#pragma unroll
  for (int db = 0; db < DB; ++db) v_addr[db] = lds_address(&sV[0][0]) + 2 * v_rd[db];

  // ---- a slot of the tile stream: one key tile of one item, with the cache-block ids its
  //      request needs (this wave's quarter of the tile, and the block of the item's frontier)
  struct Slot {
    int kt, ke, kvh, wg_max, seq;
    const int32_t* row;  // the stream's block-table row
    int64_t head_off;    // element offset of the kv head inside a cache row
    int id, last_id;
    int live;            // an int: a bool would leave tail padding that struct copies drag through memory
  };
  auto first_slot = [&](const i32x8& d, int seq) {
    Slot s;
    s.kt = d[5] & 0xffff; s.ke = d[5] >> 16; s.kvh = d[3] & 255; s.wg_max = d[4]; s.seq = seq;
    s.row = p.block_table + static_cast<int64_t>(d[3] >> 8) * p.max_blocks;
    s.head_off = static_cast<int64_t>(d[3] & 255) * p.stride_head;
    s.id = 0; s.last_id = 0;
    s.live = (d[5] >> 16) > 0 ? 1 : 0;
    return s;
  };
  auto successor = [&](const Slot& c) {
    if (c.kt + 1 < c.ke) {
      Slot s = c;
      s.kt = c.kt + 1;
      return s;
    }
    const int rel = c.seq + 1 - seq0;                       // 1 or 2
    return first_slot(rel == 1 ? d1 : d2, c.seq + 1);
  };
  auto request_ids = [&](Slot& s) {
    const int last_blk = max(s.wg_max, 0) >> 4;           // CS_KV_BLOCK = 16
    s.id = sload1(s.row + min(s.kt * 4 + wave, last_blk));
    s.last_id = sload1(s.row + last_blk);
  };
  // A tile request is 8 DMA instructions per wave (4 for K, 4 for V), each moving 1 KiB.  The
  // memory pipeline takes them at 64 bytes per clock, so issued back to back they hold the wave
  // for hundreds of cycles: regular tiles are issued one instruction at a time between the MFMAs
  // of the S phase instead (request_part), with a wave-uniform base in SGPRs and the lane's
  // constant 32-bit offset.  The S phase always issues its eight parts, so that no branch or
  // predicate splits the block of MFMAs: when there is nothing to request (the next tile holds a
  // frontier and went out at once, or there is no next tile) the parts re-read the current
  // tile's cache block into a 1-KiB sink.
  const uint16_t *req_k = nullptr, *req_v = nullptr;
  uint32_t req_dst_k = 0, req_dst_v = 0, req_step = 0;
  const uint32_t lds_k0 = lds_address(&sK[0][wave * IPW * 512]), lds_v0 = lds_address(&sV[0][wave * IPW * 512]);
  const uint32_t lds_sink = lds_address(&s_sink[wave][0]);
  auto request_part = [&](int part) {
    const int i = part & 3;
    if (part < 4) dma16_sa(k_off[i], req_k, req_dst_k + i * req_step);
    else dma16_sa(v_off[i], req_v, req_dst_v + i * req_step);
  };
  auto prepare_sink = [&](const Slot& s) {
    const int64_t at = s.head_off + static_cast<int64_t>(static_cast<uint64_t>(static_cast<uint32_t>(s.id)) *
                                                         static_cast<uint32_t>(blk_stride));
    req_k = kall + at;
    req_v = vall + at;
    req_dst_k = req_dst_v = lds_sink;
    req_step = 0;
  };
  auto prepare_regular = [&](const Slot& s, int stage) {
    // (a block spans fewer than 2^31 elements: the host checks the slot stride)
    const int64_t at = s.head_off + static_cast<int64_t>(static_cast<uint64_t>(static_cast<uint32_t>(s.id)) *
                                                         static_cast<uint32_t>(blk_stride));
    req_k = kall + at;
    req_v = vall + at;
    req_dst_k = lds_k0 + stage * (TILE * 2);
    req_dst_v = lds_v0 + stage * (TILE * 2);
    req_step = 1024;
  };
  auto issue_frontier = [&](const Slot& s, int stage) {
    // the tile that holds the frontier of its item (one per item, issued at once): rows past the
    // frontier may be unallocated or hold anything, they fetch the frontier row instead (finite
    // data, weight 0 after masking)
    const uint16_t* kg = kall + s.head_off;
    const uint16_t* vg = vall + s.head_off;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int q = wave * IPW + i;
      const int j_un = s.kt * kBN + 4 * q + l_row;
      const bool over = j_un > s.wg_max;
      const int j = over ? s.wg_max : j_un;
      const int64_t slot = static_cast<int64_t>(over ? s.last_id : s.id) * CS_KV_BLOCK + j % CS_KV_BLOCK;
      dma16(kg + slot * p.stride_slot + k_chunk[i] * 8, &sK[stage][q * 512]);
      dma16(vg + slot * p.stride_slot + v_chunk[i] * 8, &sV[stage][q * 512]);
    }
  };
  auto issue = [&](const Slot& s, int stage) {     // the whole request at once
    if (s.kt != s.wg_max / kBN) {
      prepare_regular(s, stage);
#pragma unroll
      for (int part = 0; part < 2 * IPW; ++part) request_part(part);
    } else {
      issue_frontier(s, stage);
    }
  };

  // ---- per-item state of the lane
  bf16x8 qf[RB][STEPS];
  int lim_raw[RB];
  int it_tok_head[RB], it_part = -1;
  bool it_valid[RB];
  int it_rows_left = 0;                 // rows of the stream at and after this wave's first row
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    lim_raw[rb] = 0;
    it_tok_head[rb] = 0;
    it_valid[rb] = false;
  }
  auto load_item = [&](const i32x8& d) {
    it_part = d[7];
    it_rows_left = d[1] - (d[2] + wave * WROWS);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int row = d[2] + wave * WROWS + rb * 32 + n;
      it_valid[rb] = row < d[1];
      const int row_c = it_valid[rb] ? row : d[1] - 1;
      const int tq = row_c / p.group;
      const int tok = d[0] + tq;
      it_tok_head[rb] = tok * p.n_q_heads + (d[3] & 255) * p.group + (row_c - tq * p.group);
      const uint16_t* qrow = static_cast<const uint16_t*>(p.q) + static_cast<int64_t>(it_tok_head[rb]) * D;
#pragma unroll
      for (int st = 0; st < STEPS; ++st)
        qf[rb][st] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const cs::u32x4*>(qrow + 16 * st + 8 * h));
      lim_raw[rb] = min(p.q_pos[tok], d[4]);      // d[4]: the tile's frontier, already inside the stream's entries
    }
  };

  f32x16 o[RB][DB];
  float m_run[RB], l_run[RB];
  int lim[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[rb][db][r] = 0.f;
    m_run[rb] = kNegInf;
    l_run[rb] = 0.f;
    lim[rb] = -1;
  }
  const float slack = kMaxSlack / p.scale_log2e;
  int wave_min = -1, wave_max = -1;

  auto compute = [&](int kt, int stage) {
    const int j0 = kt * kBN;
    f32x16 sacc[RB][2];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    constexpr int KPF = 2;        // K fragments are read two steps ahead of their MFMAs
    bf16x8 ka[KPF + 1][2];
    typedef __attribute__((address_space(3))) const cs::u32x4 lds_u32x4;
    // LDS addresses of this tile's fragments: one add per address and tile; pinning them in
    // registers lets every read fold its row-group offset into the instruction's immediate field
    // (formed at each use they cost two vector instructions per pair of reads)
    const uint32_t stage_off = static_cast<uint32_t>(stage) * (TILE * 2);
    uint32_t kad[STEPS], va[DB];
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      kad[st] = k_addr[st] + stage_off;
      asm volatile("" : "+v"(kad[st]));
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      va[db] = v_addr[db] + stage_off;
      asm volatile("" : "+v"(va[db]));
    }
    auto k_frag = [&](int st, int kb) {
      return __builtin_bit_cast(bf16x8, reinterpret_cast<lds_u32x4*>(static_cast<uintptr_t>(kad[st]))[kb * 32 * D * 2 / 16]);
    };
#pragma unroll
    for (int st = 0; st < KPF; ++st) {
      ka[st][0] = k_frag(st, 0);
      ka[st][1] = k_frag(st, 1);
    }
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      if (st + KPF < STEPS) {
        ka[(st + KPF) % (KPF + 1)][0] = k_frag(st + KPF, 0);
        ka[(st + KPF) % (KPF + 1)][1] = k_frag(st + KPF, 1);
      }
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          sacc[rb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[st % (KPF + 1)][kb], qf[rb][st],
                                                                 st == 0 ? zero16 : sacc[rb][kb], 0, 0, 0);
      request_part(st);
    }
    // pin that order (the scheduler would otherwise pull each read back to just before its use)
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * KPF, 0);
#pragma unroll
    for (int st = 0; st < STEPS - KPF; ++st) {
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * RB, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * RB * KPF, 0);
    bf16x8 pb[RB][2][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if (j0 + kBN - 1 > wave_min) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = j0 + 32 * kb + 8 * (r / 4) + 4 * h + (r % 4);
            if (key > lim[rb]) sacc[rb][kb][r] = kNegInf;
          }
      }
      float t_max = kNegInf;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) t_max = fmaxf(t_max, sacc[rb][kb][r]);
      {
        // the two half-waves hold the same queries: v_permlane32_swap hands each half the other's
        // value (no trip through LDS as a cross-lane shuffle would take)
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(t_max), __float_as_uint(t_max), false, false);
        t_max = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
      }
      if (__any(t_max > m_run[rb] + slack)) {
        const bool up = t_max > m_run[rb] + slack;
        const float m_new = up ? t_max : m_run[rb];
        const float alpha = up ? __builtin_amdgcn_exp2f((m_run[rb] - m_new) * p.scale_log2e) : 1.f;
        m_run[rb] = m_new;
        l_run[rb] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[rb][db][r] *= alpha;
      }
      const float m_scaled = (m_run[rb] == kNegInf ? 0.f : m_run[rb]) * p.scale_log2e;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          cs::u32x4 w;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const float e0 = __builtin_amdgcn_exp2f(fmaf(sacc[rb][kb][8 * mm + 2 * c], p.scale_log2e, -m_scaled));
            const float e1 = __builtin_amdgcn_exp2f(fmaf(sacc[rb][kb][8 * mm + 2 * c + 1], p.scale_log2e, -m_scaled));
            const uint32_t pk = pack_bf16x2(e0, e1);
            l_run[rb] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk),
                                                        __builtin_bit_cast(bf16x2, 0x3f803f80u), l_run[rb], false);
            w[c] = pk;
          }
          pb[rb][kb][mm] = __builtin_bit_cast(bf16x8, w);
        }
    }
    // 16 MFMAs, m = (key block, key half, d block); V^T fragments are read VPF MFMAs ahead
    constexpr int VPF = 3;
    s16x4 vlo[VPF + 1], vhi[VPF + 1];
    auto v_frag = [&](int m) {
      const int g0 = (32 * (m >> 3) + 16 * ((m >> 2) & 1)) * D, db = m & 3;
      const uint32_t a = va[db];
      vlo[m % (VPF + 1)] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(((lds_s16x4*)(static_cast<uintptr_t>(a))) + g0 * 2 / 8);
      vhi[m % (VPF + 1)] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(((lds_s16x4*)(static_cast<uintptr_t>(a))) + (g0 + 8 * D) * 2 / 8);
    };
#pragma unroll
    for (int m = 0; m < VPF; ++m) v_frag(m);
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      if (m + VPF < 16) v_frag(m + VPF);
      const s16x8 a = __builtin_shufflevector(vlo[m % (VPF + 1)], vhi[m % (VPF + 1)], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        o[rb][m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                              pb[rb][m >> 3][(m >> 2) & 1], o[rb][m & 3], 0, 0, 0);
    }
  };

  // Normalises and stores the rows of the finished item (or its un-normalised partial rows when
  // the key sweep is shared), then clears the accumulators.
  auto finish_item = [&](const int (&tok_head)[RB], const bool (&valid)[RB], int part) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float l_tot = l_run[rb] + __shfl_xor(l_run[rb], 32);
      if (part >= 0) {
        const int64_t prow = static_cast<int64_t>(part) + wave * WROWS + rb * 32 + n;
        if (h == 0) {
          p.ws_ml[prow * 2] = m_run[rb];
          p.ws_ml[prow * 2 + 1] = l_tot;
        }
        float* po = p.ws_o + prow * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const cs::u32x4 w = {__float_as_uint(o[rb][db][4 * rq + 0]), __float_as_uint(o[rb][db][4 * rq + 1]),
                                 __float_as_uint(o[rb][db][4 * rq + 2]), __float_as_uint(o[rb][db][4 * rq + 3])};
            *reinterpret_cast<cs::u32x4*>(po + 32 * db + 8 * rq + 4 * h) = w;
          }
      } else if (valid[rb]) {
        const float inv = __builtin_amdgcn_rcpf(l_tot);      // 1 ulp: far below the bf16 result's rounding
        uint16_t* orow = static_cast<uint16_t*>(p.out) + static_cast<int64_t>(tok_head[rb]) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            cs::u32x2 w;
            w.x = pack_bf16x2(o[rb][db][4 * rq + 0] * inv, o[rb][db][4 * rq + 1] * inv);
            w.y = pack_bf16x2(o[rb][db][4 * rq + 2] * inv, o[rb][db][4 * rq + 3] * inv);
            *reinterpret_cast<cs::u32x2*>(orow + 32 * db + 8 * rq + 4 * h) = w;
          }
      }
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[rb][db][r] = 0.f;
      m_run[rb] = kNegInf;
      l_run[rb] = 0.f;
    }
  };

  // ---- prologue: first item, first tile request, block ids of the second slot
  Slot cur = first_slot(d0, 0);
  cur.id = wave == 0 ? e0[4] : wave == 1 ? e0[5] : wave == 2 ? e0[6] : e0[7];
  cur.last_id = e0[3];
  issue(cur, 0);
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(d1), "+s"(d2));
  Slot nxt = successor(cur);
  request_ids(nxt);
  load_item(d0);
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(nxt.id), "+s"(nxt.last_id));
  bool new_item = true, ep_pending = false, ep_valid[RB];
  int ep_tok_head[RB], ep_part = -1;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    ep_valid[rb] = false;
    ep_tok_head[rb] = 0;
  }
  int stage = 0;

  for (;;) {
    // everything requested so far has landed: the tile of `cur`, and at an item boundary the Q
    // rows and frontier of its item (telling the compiler so here keeps it from waiting for them
    // later, when that wait would also cover the tile request issued below)
    wait_vmcnt<0>();
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
      for (int st = 0; st < STEPS; ++st) asm volatile("" : "+v"(qf[rb][st]));
      asm volatile("" : "+v"(lim_raw[rb]));
    }
    __syncthreads();                     // every wave's share landed; every wave left the other stage
    if (new_item) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) lim[rb] = it_valid[rb] ? lim_raw[rb] : -1;
      const int rows_here = min(WROWS, it_rows_left);     // rows of this wave that exist
      const int last = max(rows_here, 1) - 1;             // positions do not decrease along the rows
      wave_min = rows_here > 0 ? __builtin_amdgcn_readlane(lim[0], 0) : -1;
      wave_max = rows_here > 0 ? __builtin_amdgcn_readlane(lim[RB > 1 && last >= 32 ? RB - 1 : 0], last & 31) : -1;
      new_item = false;
    }
    // request the next tile: at once if it holds the frontier of its item or if this wave has
    // nothing to compute in this step, else spread over the S phase of this step
    const bool computes = cur.kt * kBN <= wave_max;
    if (nxt.live && computes && nxt.kt != nxt.wg_max / kBN) {
      prepare_regular(nxt, stage ^ 1);
    } else {
      if (nxt.live) issue(nxt, stage ^ 1);
      prepare_sink(cur);
    }

    // scalar requests for later steps: block ids of the slot after next; at the last tile of an
    // item also the descriptor three items ahead
    const bool cur_last = cur.kt + 1 == cur.ke;
    // (always issued, towards harmless addresses when there is nothing to fetch: a conditional
    // request would let the compiler merge the pending register with another value before the wait)
    Slot nn = nxt.live ? successor(nxt) : nxt;
    request_ids(nn);
    i32x8 d3 = sload8(cur_last ? item_at(d2[6]) : p.ws_plan + kHdrEndItem);

    if (ep_pending) {
      finish_item(ep_tok_head, ep_valid, ep_part);
      ep_pending = false;
    }
    if (computes) compute(cur.kt, stage);

    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(nn.id), "+s"(nn.last_id), "+s"(d3));
    if (cur_last) {
      ep_pending = true;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        ep_tok_head[rb] = it_tok_head[rb];
        ep_valid[rb] = it_valid[rb];
      }
      ep_part = it_part;
      if ((d1[5] >> 16) > 0) {
        load_item(d1);
        new_item = true;
      }
      d0 = d1; d1 = d2; d2 = d3;
      ++seq0;
    }
    if (!nxt.live) break;
    cur = nxt;
    nxt = nn;
    stage ^= 1;
  }
  finish_item(ep_tok_head, ep_valid, ep_part);
}

// Merges the partial results of split row tiles: out = sum_c w_c O_c / sum_c w_c l_c with
// w_c = 2^((m_c - max_c m_c) * scale * log2 e).  One workgroup per 8 rows; 32 threads per row.
__global__ __launch_bounds__(256) void window_attn_merge_kernel(AttnParams p) {
  constexpr int D = 128;
  const int groups = p.bm / 8;
  const int item = blockIdx.x / groups;              // < the row-tile capacity the grid was sized for
  const int32_t* d = p.ws_desc + item * 8;
  const int n_split = d[4];
  if (n_split <= 1) return;
  const int q0 = d[0], rows_total = d[1], r_tile = d[2], kvh = d[3];
  const int sub = threadIdx.x & 31;                    // 4 consecutive output dims
  const int rl = (blockIdx.x - item * groups) * 8 + (threadIdx.x >> 5);
  const int row = r_tile + rl;
  if (row >= rows_total) return;
  const int64_t base = (p.span ? static_cast<int64_t>(d[5]) : static_cast<int64_t>(item) * p.max_splits) * p.bm + rl;
  // one pass, four key ranges at a time: all loads of a batch are independent of each other and
  // of the running maximum (rows a range did not see hold m = -inf, l = 0, O = 0)
  float m_all = kNegInf, l_all = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int c0 = 0; c0 < n_split; c0 += 4) {
    float2 ml[4];
    float4 t[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t pr = base + static_cast<int64_t>(min(c0 + u, n_split - 1)) * p.bm;
      ml[u] = *reinterpret_cast<const float2*>(p.ws_ml + pr * 2);
      t[u] = *reinterpret_cast<const float4*>(p.ws_o + pr * D + 4 * sub);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (c0 + u >= n_split || ml[u].x == kNegInf) continue;
      const float m_new = fmaxf(m_all, ml[u].x);
      const float a = m_all == kNegInf ? 0.f : __builtin_amdgcn_exp2f((m_all - m_new) * p.scale_log2e);
      const float w = __builtin_amdgcn_exp2f((ml[u].x - m_new) * p.scale_log2e);
      m_all = m_new;
      l_all = fmaf(w, ml[u].y, l_all * a);
      acc[0] = fmaf(w, t[u].x, acc[0] * a); acc[1] = fmaf(w, t[u].y, acc[1] * a);
      acc[2] = fmaf(w, t[u].z, acc[2] * a); acc[3] = fmaf(w, t[u].w, acc[3] * a);
    }
  }
  const float inv = 1.f / l_all;
  const int tok = q0 + row / p.group;
  const int head = kvh * p.group + row % p.group;
  uint16_t* orow = static_cast<uint16_t*>(p.out) + (static_cast<int64_t>(tok) * p.n_q_heads + head) * D;
  cs::u32x2 w2;
  w2.x = pack_bf16x2(acc[0] * inv, acc[1] * inv);
  w2.y = pack_bf16x2(acc[2] * inv, acc[3] * inv);
  *reinterpret_cast<cs::u32x2*>(orow + 4 * sub) = w2;
}

// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void window_attn_f32_kernel(AttnParams p) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t unit = static_cast<int64_t>(blockIdx.x) * 4 + wave;      // (query, head)
  if (unit >= p.n_q * p.n_q_heads) return;
  const int tok = static_cast<int>(unit / p.n_q_heads);
  if (tok >= p.cu_q[p.n_streams]) return;               // n_q may be an upper bound
  const int head = static_cast<int>(unit - static_cast<int64_t>(tok) * p.n_q_heads);
  const int kvh = head / p.group;
  int s = 0;
  while (s + 1 < p.n_streams && p.cu_q[s + 1] <= tok) ++s;
  const int32_t* bt = p.block_table + static_cast<int64_t>(s) * p.max_blocks;
  const int lim = min(p.q_pos[tok], min(p.kv_len[s], p.max_blocks * CS_KV_BLOCK) - 1);
  if (lim < 0) return;                    // the stream defines no cache entry (or q_pos < 0): row left untouched

  const float* qrow = static_cast<const float*>(p.q) + (static_cast<int64_t>(tok) * p.n_q_heads + head) * D;
  float qv[D], acc[D];
#pragma unroll
  for (int c = 0; c < D; c += 4) {
    const float4 t = *reinterpret_cast<const float4*>(qrow + c);
    qv[c] = t.x; qv[c + 1] = t.y; qv[c + 2] = t.z; qv[c + 3] = t.w;
  }
#pragma unroll
  for (int c = 0; c < D; ++c) acc[c] = 0.f;
  float m = kNegInf, l = 0.f;
  const float* kb = static_cast<const float*>(p.k) + kvh * p.stride_head;
  const float* vb = static_cast<const float*>(p.v) + kvh * p.stride_head;
  for (int j = lane; j <= lim; j += 64) {
    const int64_t slot = static_cast<int64_t>(bt[j / CS_KV_BLOCK]) * CS_KV_BLOCK + j % CS_KV_BLOCK;
    const float* kr = kb + slot * p.stride_slot;
    const float* vr = vb + slot * p.stride_slot;
    float dot = 0.f;
#pragma unroll
    for (int c = 0; c < D; c += 4) {
      const float4 t = *reinterpret_cast<const float4*>(kr + c);
      dot = fmaf(qv[c], t.x, dot); dot = fmaf(qv[c + 1], t.y, dot);
      dot = fmaf(qv[c + 2], t.z, dot); dot = fmaf(qv[c + 3], t.w, dot);
    }
    const float sc = dot * p.scale;
    const float m_new = fmaxf(m, sc);
    const float a = expf(m - m_new);            // exp(-inf) = 0 on the first key
    const float w = expf(sc - m_new);
    l = fmaf(l, a, w);
#pragma unroll
    for (int c = 0; c < D; c += 4) {
      const float4 t = *reinterpret_cast<const float4*>(vr + c);
      acc[c] = fmaf(acc[c], a, w * t.x); acc[c + 1] = fmaf(acc[c + 1], a, w * t.y);
      acc[c + 2] = fmaf(acc[c + 2], a, w * t.z); acc[c + 3] = fmaf(acc[c + 3], a, w * t.w);
    }
    m = m_new;
  }
  // merge the 64 per-lane partial results
  float m_all = m;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m_all = fmaxf(m_all, __shfl_xor(m_all, off));
  const float w = m == kNegInf ? 0.f : expf(m - m_all);
  float l_all = l * w;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) l_all += __shfl_xor(l_all, off);
  const float inv = 1.f / l_all;
  float* orow = static_cast<float*>(p.out) + (static_cast<int64_t>(tok) * p.n_q_heads + head) * D;
#pragma unroll
  for (int c = 0; c < D; ++c) {
    float t = acc[c] * w;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) t += __shfl_xor(t, off);
    if (lane == (c & 63)) orow[c] = t * inv;
  }
}

// Launch shape and workspace layout of the bf16 / head_dim 128 path, shared by the workspace
// query and the call.
struct AttnPlan {
  int64_t r_cap;         // upper bound on row tiles per kv head
  int64_t rt_cap;        // ... times kv heads
  int64_t items_cap;     // upper bound on work items
  int chunk_tiles;       // key tiles per item when a row tile's sweep is split
  int max_splits, max_tiles;
  int grid;              // persistent workgroups: 8 XCDs x up to 64
  int bm;                // rows per item
  int rb;                // 32-row blocks per wave
  int hist_pitch;        // buckets of the planner's counting sort, per XCD
  int span, pref_pitch;  // span plan (see plan_spans) and the ints per XCD of its prefix array
  size_t off_pref;
  size_t off_items, off_rt_desc, off_st_toff, off_st_work, off_st_rank, off_rt_stream, off_rt_wgmax,
      off_hist, off_ml, off_o, total;
};

AttnPlan plan_attn(int64_t n_q, int32_t n_streams, int32_t group, int32_t n_kv_heads, int32_t max_blocks) {
  AttnPlan a;
  a.rb = 1;
  a.bm = kBM * a.rb;
  a.r_cap = (n_q * group) / a.bm + n_streams;
  a.rt_cap = a.r_cap * n_kv_heads;
  a.max_tiles = static_cast<int>((static_cast<int64_t>(max_blocks) * CS_KV_BLOCK + kBN - 1) / kBN);
  // split long key sweeps when the row tiles alone cannot fill the chip a couple of times over
  const int64_t target = 1024;
  a.chunk_tiles = 1 << 30;
  a.max_splits = 1;
  if (a.rt_cap < target && a.max_tiles > 4) {
    const int wanted = static_cast<int>((target + a.rt_cap - 1) / a.rt_cap);
    a.chunk_tiles = a.max_tiles / wanted;
    if (a.chunk_tiles < 4) a.chunk_tiles = 4;
    a.max_splits = (a.max_tiles + a.chunk_tiles - 1) / a.chunk_tiles;
    if (a.max_splits <= 1) { a.max_splits = 1; a.chunk_tiles = 1 << 30; }
  }
  a.span = a.max_splits > 1 ? 1 : 0;
  // span plan: every cut adds one item, and an item's list position names its partial-result slot
  a.items_cap = a.span ? a.rt_cap + 8 * kSlotsPerXcd : a.rt_cap * a.max_splits;
  a.pref_pitch = static_cast<int>(a.rt_cap / 8 + 2);
  const int64_t per_xcd = (a.items_cap + 7) / 8;
  const int64_t cap = a.rb == 2 ? 32 : 64;
  a.grid = 8 * static_cast<int>(per_xcd < cap ? per_xcd : cap);
  size_t at = kPlanHeaderInts * sizeof(int32_t);
  auto take = [&](size_t bytes) {
    const size_t here = (at + 255) & ~static_cast<size_t>(255);
    at = here + bytes;
    return here;
  };
  a.off_items = take(static_cast<size_t>(a.items_cap) * 8 * sizeof(int32_t));
  a.off_rt_desc = take(static_cast<size_t>(a.rt_cap) * 8 * sizeof(int32_t));
  a.off_st_toff = take((static_cast<size_t>(n_streams) + 1) * sizeof(int32_t));
  a.off_st_work = take(static_cast<size_t>(n_streams) * sizeof(int32_t));
  a.off_st_rank = take(static_cast<size_t>(n_streams) * sizeof(int32_t));
  a.off_rt_stream = take(static_cast<size_t>(a.r_cap) * sizeof(int32_t));
  a.off_rt_wgmax = take(static_cast<size_t>(a.r_cap) * sizeof(int32_t));
  const int64_t pair_rounds = (static_cast<int64_t>(n_streams) * n_kv_heads + 7) / 8;
  a.hist_pitch = static_cast<int>((a.max_tiles + 2 > pair_rounds ? a.max_tiles + 2 : pair_rounds) + 1);
  a.off_hist = take(static_cast<size_t>(8) * a.hist_pitch * sizeof(int32_t));
  a.off_pref = take(static_cast<size_t>(8) * a.pref_pitch * sizeof(int32_t));
  const bool split = a.max_splits > 1;
  a.off_ml = take(split ? static_cast<size_t>(a.items_cap) * a.bm * 2 * sizeof(float) : 0);
  a.off_o = take(split ? static_cast<size_t>(a.items_cap) * a.bm * 128 * sizeof(float) : 0);
  a.total = (at + 255) & ~static_cast<size_t>(255);
  return a;
}

}  // namespace

extern "C" size_t cs_window_prefill_attn_workspace(int64_t n_q, int32_t n_streams, int32_t n_q_heads,
                                                   int32_t n_kv_heads, int32_t head_dim,
                                                   int32_t max_blocks, int32_t dtype) {
  if (dtype != CS_BF16 || head_dim != 128 || n_q <= 0 || n_streams <= 0 || n_kv_heads < 1 ||
      n_q_heads < n_kv_heads || max_blocks <= 0)
    return 0;
  if (n_q_heads % n_kv_heads || n_q * n_q_heads >= (1ll << 31)) return 0;
  return plan_attn(n_q, n_streams, n_q_heads / n_kv_heads, n_kv_heads, max_blocks).total;
}

namespace {

// The attention call; with k_new != nullptr the launch first writes the new K/V rows into the cache
// (bf16 / head_dim 128: inside the same launch; other shapes: the caller has already queued the
// refresh write as a launch of its own).
// The argument checks of the attention call that need no device: an error code, CS_OK (go on), or
// kAttnNothingToDo (valid arguments, empty launch).
constexpr int kAttnNothingToDo = 1;

int attn_validate(const void* q, const void* k_cache_layer, const void* v_cache_layer,
                  const int32_t* cu_q, const int32_t* q_pos, const int32_t* kv_len,
                  const int32_t* block_table, int32_t max_blocks, int32_t block_size,
                  const void* out, int64_t n_q, int32_t n_streams, int32_t n_q_heads,
                  int32_t n_kv_heads, int32_t head_dim, int64_t stride_slot,
                  int64_t stride_head, float softmax_scale, int32_t dtype, int32_t plan_mode) {
  if (n_q < 0 || n_streams < 0 || n_q_heads < 1 || n_kv_heads < 1 || max_blocks < 0) return CS_EINVAL;
  if (stride_slot < 0 || stride_head < 0) return CS_EINVAL;
  if (n_q_heads % n_kv_heads) return CS_EINVAL;
  if (!(softmax_scale > 0.f) || !isfinite(softmax_scale)) return CS_EINVAL;   // also rejects NaN
  if (dtype != CS_F32 && dtype != CS_BF16) return CS_EUNSUPPORTED;
  if (head_dim != 64 && head_dim != 128) return CS_EUNSUPPORTED;
  if (block_size != CS_KV_BLOCK) return CS_EUNSUPPORTED;
  if (n_q_heads / n_kv_heads > 16) return CS_EUNSUPPORTED;
  const int elems = dtype == CS_BF16 ? 8 : 4;
  if (stride_slot % elems || stride_head % elems) return CS_EUNSUPPORTED;
  if (n_q == 0 || n_streams == 0) return kAttnNothingToDo;
  const bool plan_only = plan_mode == CS_ATTN_PLAN_ONLY && dtype == CS_BF16 && head_dim == 128;
  if (!cu_q || !q_pos || !kv_len || !block_table) return CS_EINVAL;
  if (!plan_only && (!q || !k_cache_layer || !v_cache_layer || !out)) return CS_EINVAL;
  if (!cs::aligned16(q) || !cs::aligned16(out) || !cs::aligned16(k_cache_layer) ||
      !cs::aligned16(v_cache_layer))
    return CS_EUNSUPPORTED;
  if (n_q * n_q_heads >= (1ll << 31)) return CS_EUNSUPPORTED;
  if (dtype == CS_BF16 && head_dim == 64 && max_blocks > kMaxBlocksInLds) return CS_EUNSUPPORTED;
  return CS_OK;
}

int attn_call(const void* q, const void* k_cache_layer, const void* v_cache_layer,
              const int32_t* cu_q, const int32_t* q_pos, const int32_t* kv_len,
              const int32_t* block_table, int32_t max_blocks, int32_t block_size,
              void* out, int64_t n_q, int32_t n_streams, int32_t n_q_heads,
              int32_t n_kv_heads, int32_t head_dim, int64_t stride_slot,
              int64_t stride_head, float softmax_scale, int32_t dtype,
              void* workspace, size_t workspace_bytes, int32_t plan_mode,
              const void* k_new, const void* v_new, const int32_t* new_slot, int64_t n_new,
              void* stream) {
  const int checked = attn_validate(q, k_cache_layer, v_cache_layer, cu_q, q_pos, kv_len, block_table, max_blocks,
                                    block_size, out, n_q, n_streams, n_q_heads, n_kv_heads, head_dim, stride_slot,
                                    stride_head, softmax_scale, dtype, plan_mode);
  if (checked == kAttnNothingToDo) return CS_OK;
  if (checked != CS_OK) return checked;
  const int group = n_q_heads / n_kv_heads;

  AttnParams p;
  p.q = q;
  p.k = k_cache_layer;
  p.v = v_cache_layer;
  p.out = out;
  p.cu_q = cu_q;
  p.q_pos = q_pos;
  p.block_table = block_table;
  p.kv_len = kv_len;
  p.stride_slot = stride_slot;
  p.stride_head = stride_head;
  p.max_blocks = max_blocks;
  p.n_streams = n_streams;
  p.n_q_heads = n_q_heads;
  p.n_kv_heads = n_kv_heads;
  p.group = group;
  p.scale = softmax_scale;
  p.scale_log2e = softmax_scale * 1.4426950408889634f;
  p.n_q = n_q;
  const bool fuse = k_new != nullptr;
  p.k_new = k_new;
  p.v_new = v_new;
  p.new_slot = new_slot;
  p.n_new = n_new;
  p.head_vecs = head_dim / 8;
  p.row_vecs = n_kv_heads * p.head_vecs;
  p.ws_sync = nullptr;
  p.ws_status = nullptr;
  hipStream_t st = cs::as_stream(stream);
  if (dtype == CS_BF16) {
    const size_t bt_bytes = static_cast<size_t>(max_blocks) * sizeof(int32_t);
    if (head_dim == 128) {
      if (n_kv_heads > 256 || n_streams >= (1 << 23)) return CS_EUNSUPPORTED;
      if (plan_mode != CS_ATTN_PLAN_BUILD && plan_mode != CS_ATTN_PLAN_REUSE && plan_mode != CS_ATTN_PLAN_ONLY)
        return CS_EINVAL;
      const AttnPlan a = plan_attn(n_q, n_streams, group, n_kv_heads, max_blocks);
      if (a.items_cap * a.bm >= (1ll << 31)) return CS_EUNSUPPORTED;
      if (stride_slot >= (1ll << 26) || a.max_tiles >= (1 << 15)) return CS_EUNSUPPORTED;      // 32-bit byte offsets inside a cache block
      if (!workspace || workspace_bytes < a.total || !cs::aligned16(workspace)) return CS_EWORKSPACE;
      char* w = static_cast<char*>(workspace);
      p.bm = a.bm;
      p.chunk_tiles = a.chunk_tiles;
      p.max_splits = a.max_splits;
      p.span = a.span;
      p.ws_plan = reinterpret_cast<const int32_t*>(w);
      p.ws_sync = reinterpret_cast<int32_t*>(w) + kHdrSyncBase;
      p.ws_status = reinterpret_cast<int32_t*>(w) + kHdrStatus;
      p.ws_items = reinterpret_cast<const int32_t*>(w + a.off_items);
      p.ws_desc = reinterpret_cast<int32_t*>(w + a.off_rt_desc);
      p.ws_ml = reinterpret_cast<float*>(w + a.off_ml);
      p.ws_o = reinterpret_cast<float*>(w + a.off_o);
      if (plan_mode != CS_ATTN_PLAN_REUSE) {
        PlanParams pp;
        pp.cu_q = cu_q;
        pp.q_pos = q_pos;
        pp.block_table = block_table;
        pp.kv_len = kv_len;
        pp.max_blocks = max_blocks;
        pp.n_streams = n_streams;
        pp.group = group;
        pp.n_kv_heads = n_kv_heads;
        pp.chunk_tiles = a.chunk_tiles;
        pp.max_splits = a.max_splits;
        pp.max_tiles = a.max_tiles;
        pp.r_cap = static_cast<int32_t>(a.r_cap);
        pp.bm = a.bm;
        pp.n_slots = a.grid / 8;
        pp.hist_pitch = a.hist_pitch;
        pp.header = reinterpret_cast<int32_t*>(w);
        pp.items = reinterpret_cast<int32_t*>(w + a.off_items);
        pp.rt_desc = reinterpret_cast<int32_t*>(w + a.off_rt_desc);
        pp.st_toff = reinterpret_cast<int32_t*>(w + a.off_st_toff);
        pp.st_work = reinterpret_cast<int32_t*>(w + a.off_st_work);
        pp.st_rank = reinterpret_cast<int32_t*>(w + a.off_st_rank);
        pp.rt_stream = reinterpret_cast<int32_t*>(w + a.off_rt_stream);
        pp.rt_wgmax = reinterpret_cast<int32_t*>(w + a.off_rt_wgmax);
        pp.hist = reinterpret_cast<int32_t*>(w + a.off_hist);
        pp.span = a.span;
        pp.pref_pitch = a.pref_pitch;
        pp.sw_pref = reinterpret_cast<int32_t*>(w + a.off_pref);
        hipLaunchKernelGGL(window_attn_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, pp);
        const int e = cs::note_hip(hipGetLastError());
        if (e != CS_OK) return e;
        if (plan_mode == CS_ATTN_PLAN_ONLY) return CS_OK;
      }
      if (fuse)
        hipLaunchKernelGGL((window_attn_bf16_stream_kernel<1, true>), dim3(static_cast<unsigned>(a.grid)), dim3(256), 0, st, p);
      else
        hipLaunchKernelGGL((window_attn_bf16_stream_kernel<1, false>), dim3(static_cast<unsigned>(a.grid)), dim3(256), 0, st, p);
      if (a.max_splits > 1) {
        const int e = cs::note_hip(hipGetLastError());
        if (e != CS_OK) return e;
        hipLaunchKernelGGL(window_attn_merge_kernel, dim3(static_cast<unsigned>(a.rt_cap * (a.bm / 8))),
                           dim3(256), 0, st, p);
      }
    } else {
      if (max_blocks > kMaxBlocksInLds) return CS_EUNSUPPORTED;
      const int64_t tiles = (n_q * group) / kBM + n_streams;           // upper bound on row tiles
      if (tiles > 0x7fffffffll) return CS_EUNSUPPORTED;
      const dim3 grid(static_cast<unsigned>(tiles), static_cast<unsigned>(n_kv_heads));
      hipLaunchKernelGGL(window_attn_bf16_kernel<64>, grid, dim3(256), bt_bytes, st, p);
    }
  } else {
    const int64_t units = n_q * n_q_heads;
    const dim3 grid(static_cast<unsigned>((units + 3) / 4));
    if (head_dim == 128)
      hipLaunchKernelGGL(window_attn_f32_kernel<128>, grid, dim3(256), 0, st, p);
    else
      hipLaunchKernelGGL(window_attn_f32_kernel<64>, grid, dim3(256), 0, st, p);
  }
  return cs::note_hip(hipGetLastError());
}

}  // namespace

extern "C" int cs_window_prefill_attn(const void* q, const void* k_cache_layer, const void* v_cache_layer,
                                      const int32_t* cu_q, const int32_t* q_pos, const int32_t* kv_len,
                                      const int32_t* block_table, int32_t max_blocks, int32_t block_size,
                                      void* out, int64_t n_q, int32_t n_streams, int32_t n_q_heads,
                                      int32_t n_kv_heads, int32_t head_dim, int64_t stride_slot,
                                      int64_t stride_head, float softmax_scale, int32_t dtype,
                                      void* workspace, size_t workspace_bytes, int32_t plan_mode,
                                      void* stream) {
  return attn_call(q, k_cache_layer, v_cache_layer, cu_q, q_pos, kv_len, block_table, max_blocks, block_size, out,
                   n_q, n_streams, n_q_heads, n_kv_heads, head_dim, stride_slot, stride_head, softmax_scale, dtype,
                   workspace, workspace_bytes, plan_mode, nullptr, nullptr, nullptr, 0, stream);
}

extern "C" int cs_refresh_prefill_attn(const void* k_new, const void* v_new, const int32_t* slot, int64_t n_tok,
                                       const void* q, void* k_cache_layer, void* v_cache_layer,
                                       const int32_t* cu_q, const int32_t* q_pos, const int32_t* kv_len,
                                       const int32_t* block_table, int32_t max_blocks, int32_t block_size,
                                       void* out, int64_t n_q, int32_t n_streams, int32_t n_q_heads,
                                       int32_t n_kv_heads, int32_t head_dim, int64_t stride_slot,
                                       int64_t stride_head, float softmax_scale, int32_t dtype,
                                       void* workspace, size_t workspace_bytes, int32_t plan_mode,
                                       void* stream) {
  if (n_tok < 0) return CS_EINVAL;
  const bool one_launch = dtype == CS_BF16 && head_dim == 128;
  const bool plan_only = plan_mode == CS_ATTN_PLAN_ONLY && one_launch;
  if (n_tok > 0 && !plan_only && (!k_new || !v_new || !slot)) return CS_EINVAL;
  if (!cs::aligned16(k_new) || !cs::aligned16(v_new)) return CS_EUNSUPPORTED;
  if (!one_launch || n_tok == 0 || n_q == 0 || n_streams == 0) {
    // shapes without a persistent kernel (fp32 caches, head_dim 64), or nothing to attend: the
    // refresh write as a launch of its own, then the attention call (whose arguments are checked
    // first, so that a call that fails has moved nothing)
    const int checked = attn_validate(q, k_cache_layer, v_cache_layer, cu_q, q_pos, kv_len, block_table, max_blocks,
                                      block_size, out, n_q, n_streams, n_q_heads, n_kv_heads, head_dim, stride_slot,
                                      stride_head, softmax_scale, dtype, plan_mode);
    if (checked < 0) return checked;
    if (n_tok > 0) {
      const int e = cs_kv_refresh_scatter(k_new, v_new, slot, k_cache_layer, v_cache_layer, n_tok, n_kv_heads,
                                          head_dim, stride_slot, stride_head, dtype, stream);
      if (e != CS_OK) return e;
    }
    return attn_call(q, k_cache_layer, v_cache_layer, cu_q, q_pos, kv_len, block_table, max_blocks, block_size, out,
                     n_q, n_streams, n_q_heads, n_kv_heads, head_dim, stride_slot, stride_head, softmax_scale, dtype,
                     workspace, workspace_bytes, plan_mode, nullptr, nullptr, nullptr, 0, stream);
  }
  return attn_call(q, k_cache_layer, v_cache_layer, cu_q, q_pos, kv_len, block_table, max_blocks, block_size, out,
                   n_q, n_streams, n_q_heads, n_kv_heads, head_dim, stride_slot, stride_head, softmax_scale, dtype,
                   workspace, workspace_bytes, plan_mode, k_new, v_new, slot, n_tok, stream);
}
