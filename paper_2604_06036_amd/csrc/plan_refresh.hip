// Refresh plan on the device.  Paper Sec. 3.4.1 (GOP-guided anchor refresh: overlap I-frames are
// recomputed, the other overlap frames are reused, new frames and the text suffix are prefilled)
// and Sec. 3.5 (planning is separated from KV-context preparation; a frame-aware index maps
// visual-token spans to physical cache slots across cache-block boundaries).
//
// Input is what the previous step and the scoring call left in device memory (frame types and
// kept-token counts of the cached window, the new frames' types, the kept-token offsets of the
// new frames, both block tables); output is every row list the later calls consume.  Nothing
// comes back to the host, so the calls of one step can be queued without a synchronisation.
//
// Three launches:
//   1. plan_frames_kernel   one wave per stream: the new window's (type, count) per frame, prefix
//                           sums over its frames (sequence start, start inside the stream's reused
//                           rows or executed rows), per-stream totals.
//   2. plan_streams_kernel  one workgroup: prefix sums of the per-stream totals over the streams
//                           (reused-row base, cu_q), grand totals, capacity flags.
//   3. plan_fill_kernel     one wave per (stream, frame) and one for the text suffix: the wave's
//                           tokens are consecutive in the sequence and consecutive in their output
//                           list, so every store is coalesced; the tail of the workgroups pads the
//                           lists up to their capacities.
// A reused token's row in the previous window is its new sequence index plus the kept-token count
// of the frames that left the window (the overlap keeps its order), so no second prefix sum over
// the old window is needed.
#include "common.h"

namespace {

constexpr int kKindAnchor = 0, kKindNew = 1, kKindText = 2, kKindReuse = 3;
constexpr int kFlagReuseCap = 1, kFlagQueryCap = 2, kFlagBlockTable = 4;

struct PlanRefreshParams {
  const uint8_t* __restrict__ old_types;     // [B][W]
  const int32_t* __restrict__ old_counts;    // [B][W]
  const uint8_t* __restrict__ new_types;     // [B][S]
  const int32_t* __restrict__ kept_off;      // [B*S + 1]
  const int32_t* __restrict__ bt_old;        // [B][max_blocks_old]
  const int32_t* __restrict__ bt_new;        // [B][max_blocks_new]
  int32_t max_blocks_old, max_blocks_new;
  int32_t n_streams, window, stride, n_text, shift;
  int64_t reuse_cap, q_cap;
  int32_t* __restrict__ src_slot;
  int32_t* __restrict__ dst_slot;
  int32_t* __restrict__ delta;
  int32_t* __restrict__ q_pos;
  int32_t* __restrict__ q_slot;
  uint8_t* __restrict__ q_kind;
  int32_t* __restrict__ cu_q;                // [B+1]
  int32_t* __restrict__ kv_len;              // [B]
  uint8_t* __restrict__ out_types;           // [B][W]
  int32_t* __restrict__ out_counts;          // [B][W]
  int32_t* __restrict__ totals;              // [4]
  // workspace
  int4* __restrict__ rec;                    // [B][W+1]: {sequence start, start in list, count, kind}
  int32_t* __restrict__ st_reuse;            // [B] reused rows of the stream
  int32_t* __restrict__ st_q;                // [B] executed rows of the stream (text included)
  int32_t* __restrict__ st_head;             // [B] kept tokens of the frames that left the window
  int32_t* __restrict__ reuse_base;          // [B]
  int32_t* __restrict__ q_base;              // [B] first executed row of the stream (cu_q before clamping)
};

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_up(v, off);
    if (lane >= off) v += t;
  }
  return v;
}

__global__ __launch_bounds__(256) void plan_frames_kernel(PlanRefreshParams p) {
  const int lane = threadIdx.x & 63;
  const int s = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= p.n_streams) return;
  const int W = p.window, S = p.stride, keep = W - S;
  const uint8_t* ot = p.old_types + static_cast<int64_t>(s) * W;
  const int32_t* oc = p.old_counts + static_cast<int64_t>(s) * W;
  const uint8_t* nt = p.new_types + static_cast<int64_t>(s) * S;
  const int32_t* ko = p.kept_off + static_cast<int64_t>(s) * S;
  int4* rec = p.rec + static_cast<int64_t>(s) * (W + 1);

  // kept tokens of the S frames that leave the window
  int head = 0;
  for (int f = lane; f < S; f += 64) head += oc[f];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) head += __shfl_xor(head, off);

  int seq_run = 0, reuse_run = 0, q_run = 0;
  for (int f0 = 0; f0 < W; f0 += 64) {
    const int f = f0 + lane;
    int type = 0, cnt = 0, kind = kKindNew;
    if (f < keep) {
      type = ot[f + S];
      cnt = oc[f + S];
      kind = type == CS_FRAME_I ? kKindAnchor : kKindReuse;
    } else if (f < W) {
      type = nt[f - keep];
      cnt = ko[f - keep + 1] - ko[f - keep];
    }
    const int c_reuse = kind == kKindReuse ? cnt : 0;
    const int c_q = cnt - c_reuse;
    const int seq_inc = wave_inclusive_scan(cnt, lane);
    const int reuse_inc = wave_inclusive_scan(c_reuse, lane);
    const int q_inc = wave_inclusive_scan(c_q, lane);
    if (f < W) {
      const int start = kind == kKindReuse ? reuse_run + reuse_inc - c_reuse : q_run + q_inc - c_q;
      rec[f] = make_int4(seq_run + seq_inc - cnt, start, cnt, kind);
      p.out_types[static_cast<int64_t>(s) * W + f] = static_cast<uint8_t>(type);
      p.out_counts[static_cast<int64_t>(s) * W + f] = cnt;
    }
    seq_run += __shfl(seq_inc, 63);
    reuse_run += __shfl(reuse_inc, 63);
    q_run += __shfl(q_inc, 63);
  }
  if (lane == 0) {
    rec[W] = make_int4(seq_run, q_run, p.n_text, kKindText);
    p.kv_len[s] = seq_run + p.n_text;
    p.st_reuse[s] = reuse_run;
    p.st_q[s] = q_run + p.n_text;
    p.st_head[s] = head;
  }
}

constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void plan_streams_kernel(PlanRefreshParams p) {
  __shared__ int part_r[kScanThreads / 64], part_q[kScanThreads / 64];
  __shared__ int run_r, run_q;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { run_r = 0; run_q = 0; }
  __syncthreads();
  for (int s0 = 0; s0 < p.n_streams; s0 += kScanThreads) {
    const int s = s0 + tid;
    const int r = s < p.n_streams ? p.st_reuse[s] : 0;
    const int q = s < p.n_streams ? p.st_q[s] : 0;
    const int r_inc = wave_inclusive_scan(r, lane);
    const int q_inc = wave_inclusive_scan(q, lane);
    if (lane == 63) { part_r[wave] = r_inc; part_q[wave] = q_inc; }
    __syncthreads();
    int base_r = run_r, base_q = run_q;
    for (int w = 0; w < wave; ++w) { base_r += part_r[w]; base_q += part_q[w]; }
    if (s < p.n_streams) {
      p.reuse_base[s] = base_r + r_inc - r;
      const int first_q = base_q + q_inc - q;
      p.q_base[s] = first_q;
      // what the consumers see never points past the capacity: rows that do not fit are dropped
      // (and flagged), the rows that do are where cu_q says
      p.cu_q[s] = static_cast<int>(min(static_cast<int64_t>(first_q), p.q_cap));
    }
    __syncthreads();
    if (tid == kScanThreads - 1) { run_r = base_r + r_inc; run_q = base_q + q_inc; }
    __syncthreads();
  }
  if (tid == 0) {
    p.cu_q[p.n_streams] = static_cast<int>(min(static_cast<int64_t>(run_q), p.q_cap));
    p.totals[0] = run_r;
    p.totals[1] = run_q;
    p.totals[2] = (run_r > p.reuse_cap ? kFlagReuseCap : 0) | (run_q > p.q_cap ? kFlagQueryCap : 0);
    p.totals[3] = 0;
  }
}

__device__ __forceinline__ int slot_of(const int32_t* bt, int max_blocks, int seq, bool* bad) {
  const int b = seq / CS_KV_BLOCK;
  if (seq < 0 || b >= max_blocks) { *bad = true; return -1; }       // also: counts that are not counts
  return bt[b] * CS_KV_BLOCK + seq % CS_KV_BLOCK;
}

__global__ __launch_bounds__(256) void plan_fill_kernel(PlanRefreshParams p, int fill_blocks, int pad_r_blocks) {
  const int lane = threadIdx.x & 63;
  const int block = blockIdx.x;
  if (block >= fill_blocks) {
    // pad the lists between their totals and their capacities
    if (block < fill_blocks + pad_r_blocks) {
      const int64_t i = static_cast<int64_t>(block - fill_blocks) * 256 + threadIdx.x;
      if (i >= p.totals[0] && i < p.reuse_cap) { p.src_slot[i] = -1; p.dst_slot[i] = -1; p.delta[i] = 0; }
    } else {
      const int64_t i = static_cast<int64_t>(block - fill_blocks - pad_r_blocks) * 256 + threadIdx.x;
      if (i >= p.totals[1] && i < p.q_cap) { p.q_pos[i] = 0; p.q_slot[i] = -1; p.q_kind[i] = 0xff; }
    }
    return;
  }
  const int64_t unit = static_cast<int64_t>(block) * 4 + (threadIdx.x >> 6);
  const int per_stream = p.window + 1;
  if (unit >= static_cast<int64_t>(p.n_streams) * per_stream) return;
  const int s = static_cast<int>(unit / per_stream);
  const int4 r = p.rec[unit];
  const int seq0 = r.x, cnt = r.z, kind = r.w;
  const int32_t* btn = p.bt_new + static_cast<int64_t>(s) * p.max_blocks_new;
  bool bad = false;
  if (kind == kKindReuse) {
    const int32_t* bto = p.bt_old + static_cast<int64_t>(s) * p.max_blocks_old;
    const int head = p.st_head[s];
    const int64_t o0 = static_cast<int64_t>(p.reuse_base[s]) + r.y;
    for (int i = lane; i < cnt; i += 64) {
      const int64_t o = o0 + i;
      const int src = slot_of(bto, p.max_blocks_old, seq0 + i + head, &bad);
      const int dst = slot_of(btn, p.max_blocks_new, seq0 + i, &bad);
      if (o < p.reuse_cap) {
        // a row with either slot missing is dropped as a whole
        p.src_slot[o] = dst < 0 ? -1 : src;
        p.dst_slot[o] = src < 0 ? -1 : dst;
        p.delta[o] = p.shift;
      }
    }
  } else {
    const int64_t o0 = static_cast<int64_t>(p.q_base[s]) + r.y;
    for (int i = lane; i < cnt; i += 64) {
      const int64_t o = o0 + i;
      const int dst = slot_of(btn, p.max_blocks_new, seq0 + i, &bad);
      if (o < p.q_cap) {
        // a position the block-table row does not cover (flagged) is pulled back onto the row, so
        // that attention queued behind this plan never indexes past the table
        p.q_pos[o] = dst < 0 ? min(seq0 + i, p.max_blocks_new * CS_KV_BLOCK - 1) : seq0 + i;
        p.q_slot[o] = dst;
        p.q_kind[o] = static_cast<uint8_t>(kind);
      }
    }
  }
  if (bad) atomicOr(p.totals + 2, kFlagBlockTable);
}

inline size_t align256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

struct PlanRefreshLayout {
  size_t off_rec, off_reuse, off_q, off_head, off_base, off_qbase, total;
};

PlanRefreshLayout layout_for(int64_t n_streams, int64_t window) {
  PlanRefreshLayout l;
  size_t at = 0;
  l.off_rec = at;      at = align256(at + static_cast<size_t>(n_streams) * (window + 1) * sizeof(int4));
  l.off_reuse = at;    at = align256(at + static_cast<size_t>(n_streams) * sizeof(int32_t));
  l.off_q = at;        at = align256(at + static_cast<size_t>(n_streams) * sizeof(int32_t));
  l.off_head = at;     at = align256(at + static_cast<size_t>(n_streams) * sizeof(int32_t));
  l.off_base = at;     at = align256(at + static_cast<size_t>(n_streams) * sizeof(int32_t));
  l.off_qbase = at;    at = align256(at + static_cast<size_t>(n_streams) * sizeof(int32_t));
  l.total = at;
  return l;
}

}  // namespace

extern "C" size_t cs_plan_refresh_workspace(int32_t n_streams, int32_t window) {
  if (n_streams <= 0 || window <= 0) return 0;
  return layout_for(n_streams, window).total;
}

extern "C" int cs_plan_refresh(const uint8_t* old_types, const int32_t* old_counts,
                               const uint8_t* new_types, const int32_t* kept_off,
                               const int32_t* block_table_old, int32_t max_blocks_old,
                               const int32_t* block_table_new, int32_t max_blocks_new,
                               int32_t n_streams, int32_t window, int32_t stride, int32_t n_text,
                               int32_t tokens_per_frame, int64_t reuse_cap, int64_t q_cap,
                               int32_t* src_slot, int32_t* dst_slot, int32_t* delta,
                               int32_t* q_pos, int32_t* q_slot, uint8_t* q_kind,
                               int32_t* cu_q, int32_t* kv_len, uint8_t* out_types, int32_t* out_counts,
                               int32_t* totals, void* workspace, size_t workspace_bytes, void* stream) {
  if (n_streams < 0 || window < 1 || stride < 1 || stride > window || n_text < 0 || tokens_per_frame < 1)
    return CS_EINVAL;
  if (max_blocks_old < 0 || max_blocks_new < 0 || reuse_cap < 0 || q_cap < 0) return CS_EINVAL;
  if (n_streams > 0 && (max_blocks_old < 1 || max_blocks_new < 1)) return CS_EINVAL;
  if (!cu_q || !totals) return CS_EINVAL;
  if (n_streams > 0 && (!old_types || !old_counts || !new_types || !kept_off || !block_table_old ||
                        !block_table_new || !kv_len || !out_types || !out_counts))
    return CS_EINVAL;
  if ((reuse_cap > 0 && (!src_slot || !dst_slot || !delta)) || (q_cap > 0 && (!q_pos || !q_slot || !q_kind)))
    return CS_EINVAL;
  const int64_t units = static_cast<int64_t>(n_streams) * (static_cast<int64_t>(window) + 1);
  if (units >= (1ll << 31) || reuse_cap >= (1ll << 31) || q_cap >= (1ll << 31)) return CS_EUNSUPPORTED;
  if (static_cast<int64_t>(stride) * tokens_per_frame >= (1ll << 31)) return CS_EUNSUPPORTED;
  const size_t need = cs_plan_refresh_workspace(n_streams, window);
  if (n_streams > 0 && (!workspace || workspace_bytes < need || !cs::aligned16(workspace))) return CS_EWORKSPACE;

  PlanRefreshParams p;
  p.old_types = old_types;
  p.old_counts = old_counts;
  p.new_types = new_types;
  p.kept_off = kept_off;
  p.bt_old = block_table_old;
  p.bt_new = block_table_new;
  p.max_blocks_old = max_blocks_old;
  p.max_blocks_new = max_blocks_new;
  p.n_streams = n_streams;
  p.window = window;
  p.stride = stride;
  p.n_text = n_text;
  p.shift = -stride * tokens_per_frame;
  p.reuse_cap = reuse_cap;
  p.q_cap = q_cap;
  p.src_slot = src_slot;
  p.dst_slot = dst_slot;
  p.delta = delta;
  p.q_pos = q_pos;
  p.q_slot = q_slot;
  p.q_kind = q_kind;
  p.cu_q = cu_q;
  p.kv_len = kv_len;
  p.out_types = out_types;
  p.out_counts = out_counts;
  p.totals = totals;
  char* w = static_cast<char*>(workspace);
  const PlanRefreshLayout l = layout_for(n_streams, window);
  p.rec = reinterpret_cast<int4*>(w + l.off_rec);
  p.st_reuse = reinterpret_cast<int32_t*>(w + l.off_reuse);
  p.st_q = reinterpret_cast<int32_t*>(w + l.off_q);
  p.st_head = reinterpret_cast<int32_t*>(w + l.off_head);
  p.reuse_base = reinterpret_cast<int32_t*>(w + l.off_base);
  p.q_base = reinterpret_cast<int32_t*>(w + l.off_qbase);

  hipStream_t st = cs::as_stream(stream);
  if (n_streams > 0) {
    hipLaunchKernelGGL(plan_frames_kernel, dim3((n_streams + 3) / 4), dim3(256), 0, st, p);
    const int e = cs::note_hip(hipGetLastError());
    if (e != CS_OK) return e;
  }
  hipLaunchKernelGGL(plan_streams_kernel, dim3(1), dim3(kScanThreads), 0, st, p);
  {
    const int e = cs::note_hip(hipGetLastError());
    if (e != CS_OK) return e;
  }
  const int64_t fill_blocks = (units + 3) / 4;
  const int64_t pad_r = (reuse_cap + 255) / 256, pad_q = (q_cap + 255) / 256;
  const int64_t blocks = fill_blocks + pad_r + pad_q;
  if (blocks >= (1ll << 31)) return CS_EUNSUPPORTED;
  if (blocks > 0)
    hipLaunchKernelGGL(plan_fill_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, p,
                       static_cast<int>(fill_blocks), static_cast<int>(pad_r));
  return cs::note_hip(hipGetLastError());
}
