// (a) Change scoring + ordered token compaction for gfx950.
//
// Paper Sec. 3.3.1-3.3.2: Eq. 1 (motion magnitude), Eq. 3-5 (retention rules), GOP accumulation,
// projection-group layout adapter, order-preserving selection of the retained tokens.
//
// Work decomposition.  The accumulated mask makes frames of one stream sequentially dependent
// but every token location is independent, so one wavefront owns one stream: its 64 lanes sweep
// the token grid 256 locations at a time (4 coalesced 4-byte metadata loads in flight per lane)
// and walk the stream's frames in temporal order.  A workgroup (4 waves = 4 consecutive streams,
// or 4 runs of up to 63 consecutive streams for batches of many thousand streams, sized so that
// all tiles are resident at once) is one tile of
// a single-pass ordered compaction:
//   pass 1  score, write keep bytes and the accumulated state, count kept tokens by ballot;
//   link    the tile publishes its count and obtains the number of tokens kept by all earlier
//           tiles through a decoupled look-back over 64-bit (flag | value) words; tiles are
//           numbered by an atomic ticket taken when the workgroup starts, so a tile only ever
//           waits for tiles that are already running;
//   pass 2  take the ballot words of pass 1 back from LDS (or, past 128 words per wave, re-read
//           the wave's own keep bytes), rank kept tokens inside each 64-token group with mbcnt,
//           and write their dense ids at base + rank.
// The look-back wait is bounded: after kSpinLimit polls a tile raises the error word in the
// workspace and continues with a zero prefix, so every wave always exits.
#include <mutex>

#include "common.h"

namespace {

constexpr int kWavesPerTile = 4;
constexpr int kGroupsPerSweep = 4;                       // 64-token groups per lane sweep
constexpr int kSweep = cs::kWave * kGroupsPerSweep;      // token locations per sweep
constexpr uint64_t kFlagAggregate = 1ull << 62;
constexpr uint64_t kFlagPrefix = 1ull << 63;
constexpr uint32_t kSpinLimit = 1u << 24;
constexpr int kEmitAhead = 4;                            // sweeps whose keep words the emit launch requests ahead
constexpr int kMaskWords = 128;                          // ballot words a wave keeps in LDS between the passes

struct ScoreParams {
  const uint32_t* __restrict__ mv;       // (dx, dy) int16 pairs viewed as one 32-bit word
  const uint32_t* __restrict__ sad;
  const uint8_t* __restrict__ intra;
  const uint8_t* __restrict__ frame_type;
  const int32_t* __restrict__ cu_frames;
  uint8_t* __restrict__ acc;
  uint8_t* __restrict__ keep;
  int32_t* __restrict__ kept_idx;
  int32_t* __restrict__ kept_off;
  uint32_t* ticket;                      // workspace word 0
  uint32_t* error;                       // workspace word 1 (second half of the first 8 bytes)
  uint64_t* tile_state;                  // workspace + 8 (one-launch form)
  uint32_t* wg_total;                    // workspace + 8 (three-launch form): kept tokens per workgroup, then their exclusive prefix
  uint32_t* wave_total;                  // ... followed by the kept tokens per wave
  int32_t n_streams, n_frames, grid_w, tok_w, n_patch, n_tok;
  int32_t streams_per_wave;              // consecutive streams swept by one wave (1 for small batches)
  int32_t single_tile;                   // one-launch form with one workgroup: no ticket, no look-back, no clearing launch
  uint32_t tau_mv_sq, tau_sad;
  int32_t use_residual;
};

__global__ void clear_words_kernel(uint64_t* w, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) w[i] = 0;
}

__global__ void zero_offsets_kernel(int32_t* off, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) off[i] = 0;
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// Patch index of sub-patch (a, b) of token t.
template <int G>
__device__ __forceinline__ int patch_of(const ScoreParams& p, int t, int a, int b) {
  if (G == 1) return t;
  const int r = t / p.tok_w, c = t - r * p.tok_w;
  return (G * r + a) * p.grid_w + G * c + b;
}

// One sweep of pass 1: 256 token locations of one frame of one stream (wave-uniform fields).
struct Sweep {
  int i;          // which of the wave's streams
  int s, f, t0;   // stream, frame, first token location
  bool is_i;
};

// What a sweep reads: metadata words (read-only inputs) and the accumulated state.
template <int G>
struct SweepRegs {
  uint32_t mvw[kGroupsPerSweep][G * G], sdw[kGroupsPerSweep][G * G];
  uint8_t inw[kGroupsPerSweep][G * G], acw[kGroupsPerSweep][G * G];
};

// PK (packed): group == 1 and a patch count that is a multiple of 4.  A lane then owns four
// CONSECUTIVE token locations of the sweep, so that its metadata are one 16-byte load per array and
// its keep / state bytes one dword each: sub-dword accesses cost the memory pipeline as much as full
// ones, and with one byte per lane they were what bounded the kernel.  Index k of the register
// arrays is then the lane's k-th location, not the k-th 64-token group.
template <int G, bool PK>
__device__ __forceinline__ void load_inputs(const ScoreParams& p, const Sweep& w, int lane, SweepRegs<G>& r) {
  constexpr int Q = G * G;
  if (w.is_i) return;                                  // an I-frame's metadata is not read
  const size_t pbase = static_cast<size_t>(w.f) * p.n_patch;
  if constexpr (PK) {
    const int t = w.t0 + 4 * lane;
    const bool valid = t < p.n_tok;
    cs::u32x4 m = {0u, 0u, 0u, 0u}, d = {0u, 0u, 0u, 0u};
    uint32_t in4 = 0u;
    if (valid) {
      m = __builtin_nontemporal_load(reinterpret_cast<const cs::u32x4*>(p.mv + pbase + t));
      if (p.use_residual) d = __builtin_nontemporal_load(reinterpret_cast<const cs::u32x4*>(p.sad + pbase + t));
      if (p.intra) in4 = *reinterpret_cast<const uint32_t*>(p.intra + pbase + t);
    }
    r.mvw[0][0] = m.x; r.mvw[1][0] = m.y; r.mvw[2][0] = m.z; r.mvw[3][0] = m.w;
    r.sdw[0][0] = d.x; r.sdw[1][0] = d.y; r.sdw[2][0] = d.z; r.sdw[3][0] = d.w;
#pragma unroll
    for (int k = 0; k < 4; ++k) r.inw[k][0] = static_cast<uint8_t>(in4 >> (8 * k));
    return;
  }
#pragma unroll
  for (int k = 0; k < kGroupsPerSweep; ++k) {
    const int t = w.t0 + k * cs::kWave + lane;
    const bool valid = t < p.n_tok;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      const int pi = valid ? patch_of<G>(p, t, q / G, q % G) : 0;
      r.mvw[k][q] = valid ? p.mv[pbase + pi] : 0u;
      r.sdw[k][q] = (valid && p.use_residual) ? p.sad[pbase + pi] : 0u;
      r.inw[k][q] = (valid && p.intra) ? p.intra[pbase + pi] : uint8_t(0);
    }
  }
}

template <int G, bool PK>
__device__ __forceinline__ void load_acc(const ScoreParams& p, const Sweep& w, int lane, SweepRegs<G>& r) {
  constexpr int Q = G * G;
  if (w.is_i || !p.acc) return;                        // an I-frame resets the state without reading it
  const uint8_t* __restrict__ acc = p.acc + static_cast<size_t>(w.s) * p.n_patch;
  if constexpr (PK) {
    const int t = w.t0 + 4 * lane;
    const uint32_t a4 = t < p.n_tok ? *reinterpret_cast<const uint32_t*>(acc + t) : 0u;
#pragma unroll
    for (int k = 0; k < 4; ++k) r.acw[k][0] = static_cast<uint8_t>(a4 >> (8 * k));
    return;
  }
#pragma unroll
  for (int k = 0; k < kGroupsPerSweep; ++k) {
    const int t = w.t0 + k * cs::kWave + lane;
#pragma unroll
    for (int q = 0; q < Q; ++q) r.acw[k][q] = t < p.n_tok ? acc[patch_of<G>(p, t, q / G, q % G)] : uint8_t(0);
  }
}

// Scores one sweep from the registers loaded for it, writes keep bytes and the changed accumulated
// state, leaves the new accumulated state in r.acw (the next frame of the same stream takes it
// from there instead of from memory); returns the number of kept tokens (wave-uniform).
template <int G, bool PK>
__device__ __forceinline__ uint32_t score_sweep(const ScoreParams& p, const Sweep& w, int lane, SweepRegs<G>& r,
                                                uint64_t* mask_cache, int& mask_words) {
  constexpr int Q = G * G;
  uint8_t* __restrict__ keep = p.keep + static_cast<size_t>(w.f) * p.n_tok;
  uint8_t* __restrict__ acc = p.acc ? p.acc + static_cast<size_t>(w.s) * p.n_patch : nullptr;
  bool bit[kGroupsPerSweep];
  if constexpr (PK) {
    const int t = w.t0 + 4 * lane;
    const bool valid = t < p.n_tok;
    uint32_t keep4 = 0u, acc4 = 0u;
    bool changed = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      bool sel;
      if (w.is_i) {
        sel = true;                                       // an I-frame keeps everything and resets the accumulation
        changed = acc != nullptr;
        r.acw[k][0] = 0;
      } else {
        const int dx = static_cast<int16_t>(r.mvw[k][0] & 0xffffu);
        const int dy = static_cast<int16_t>(r.mvw[k][0] >> 16);
        const uint32_t m = static_cast<uint32_t>(dx * dx) + static_cast<uint32_t>(dy * dy);
        const bool d_mv = m >= p.tau_mv_sq;                                        // Eq. 3
        const bool d_res = p.use_residual && !d_mv && r.sdw[k][0] >= p.tau_sad;   // Eq. 4
        sel = d_mv || d_res || r.inw[k][0] != 0;                                   // Eq. 5
        if (acc) {
          sel = sel || r.acw[k][0] != 0;                  // selected now or earlier in this GOP
          if (sel && r.acw[k][0] == 0) { r.acw[k][0] = 1; changed = true; }
        }
      }
      bit[k] = valid && sel;
      keep4 |= (sel ? 1u : 0u) << (8 * k);
      acc4 |= static_cast<uint32_t>(r.acw[k][0]) << (8 * k);
    }
    if (valid) {
      *reinterpret_cast<uint32_t*>(keep + t) = keep4;
      if (changed) *reinterpret_cast<uint32_t*>(acc + t) = acc4;   // the lane owns all four bytes
    }
  } else
#pragma unroll
  for (int k = 0; k < kGroupsPerSweep; ++k) {
    const int t = w.t0 + k * cs::kWave + lane;
    const bool valid = t < p.n_tok;
    if (w.is_i) {
      // an I-frame keeps everything and resets the accumulation
      bit[k] = valid;
      if (valid) {
        keep[t] = 1;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
          if (acc) acc[patch_of<G>(p, t, q / G, q % G)] = 0;
          r.acw[k][q] = 0;
        }
      }
    } else {
      bool any = false;
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        const int dx = static_cast<int16_t>(r.mvw[k][q] & 0xffffu);
        const int dy = static_cast<int16_t>(r.mvw[k][q] >> 16);
        const uint32_t m = static_cast<uint32_t>(dx * dx) + static_cast<uint32_t>(dy * dy);
        const bool d_mv = m >= p.tau_mv_sq;                                        // Eq. 3
        const bool d_res = p.use_residual && !d_mv && r.sdw[k][q] >= p.tau_sad;   // Eq. 4
        const bool d = d_mv || d_res || r.inw[k][q] != 0;                          // Eq. 5
        bool sel = d;
        if (acc) {
          sel = d || r.acw[k][q] != 0;                     // selected now or earlier in this GOP
          if (valid && sel && r.acw[k][q] == 0) {
            acc[patch_of<G>(p, t, q / G, q % G)] = 1;
            r.acw[k][q] = 1;
          }
        }
        any = any || sel;
      }
      bit[k] = valid && any;
      if (valid) keep[t] = any ? 1 : 0;
    }
  }
  uint32_t count = 0;
#pragma unroll
  for (int k = 0; k < kGroupsPerSweep; ++k) {
    const uint64_t mask = __ballot(bit[k]);
    if (mask_words < kMaskWords && lane == 0) mask_cache[mask_words] = mask;   // for pass 2
    ++mask_words;
    count += __popcll(mask);
  }
  return count;
}

// Writes the dense ids of the kept tokens of frame f starting at kept_idx[base]; returns count.
// The ballot words of pass 1 come back from LDS while they fit there (no memory round trip in
// this pass); beyond that the wave re-reads its own keep bytes.
template <bool PK>
__device__ uint32_t emit_frame(const ScoreParams& p, int f, uint32_t base, int lane,
                               const uint64_t* mask_cache, int& mask_words) {
  const uint8_t* keep = p.keep + static_cast<size_t>(f) * p.n_tok;
  const int32_t id0 = f * p.n_tok;
  uint32_t count = 0;
  for (int t0 = 0; t0 < p.n_tok; t0 += kSweep) {
    if constexpr (PK) {
      // word k of a sweep: which lanes keep their k-th location.  Ids ascend with (lane, k), so a
      // location's rank is the kept locations of lower lanes plus the lane's own earlier ones.
      const int t = t0 + 4 * lane;
      uint64_t mask[4];
      if (mask_words + 4 <= kMaskWords) {
#pragma unroll
        for (int k = 0; k < 4; ++k) mask[k] = mask_cache[mask_words + k];
      } else {
        const uint32_t k4 = t < p.n_tok ? *reinterpret_cast<const uint32_t*>(keep + t) : 0u;
#pragma unroll
        for (int k = 0; k < 4; ++k) mask[k] = __ballot(((k4 >> (8 * k)) & 0xffu) != 0);
      }
      mask_words += 4;
      uint32_t rank = 0, total = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        rank += lanes_below(mask[k]);
        total += __popcll(mask[k]);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if ((mask[k] >> lane) & 1) {
          p.kept_idx[base + count + rank] = id0 + t + k;
          ++rank;
        }
      }
      count += total;
      continue;
    }
#pragma unroll
    for (int k = 0; k < kGroupsPerSweep; ++k) {
      const int t = t0 + k * cs::kWave + lane;
      uint64_t mask;
      if (mask_words < kMaskWords) {
        mask = mask_cache[mask_words];
      } else {
        mask = __ballot(t < p.n_tok && keep[t] != 0);
      }
      ++mask_words;
      if ((mask >> lane) & 1) p.kept_idx[base + count + lanes_below(mask)] = id0 + t;
      count += __popcll(mask);
    }
  }
  return count;
}

// Exclusive prefix of tile `tile` over all earlier tiles (called by one full wave).  Flag and value
// travel in one 64-bit word, so relaxed device-scope atomics suffice: nothing else has to be
// ordered against them, and acquire/release here would cost an L2 invalidate / write-back per poll
// (measured: 2.4x slower on a 150k-stream batch).
__device__ uint32_t look_back(const ScoreParams& p, uint32_t tile, uint32_t aggregate, int lane) {
  if (tile == 0) {
    if (lane == 0)
      __hip_atomic_store(&p.tile_state[0], kFlagPrefix | aggregate, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    return 0;
  }
  if (lane == 0)
    __hip_atomic_store(&p.tile_state[tile], kFlagAggregate | aggregate, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
  uint32_t exclusive = 0;
  int64_t first = static_cast<int64_t>(tile) - 1;       // nearest predecessor of this window
  uint32_t polls = 0;
  for (;;) {
    const int64_t idx = first - lane;
    uint64_t st = kFlagPrefix;                            // before tile 0: prefix 0
    bool ready;
    do {
      if (idx >= 0)
        st = __hip_atomic_load(&p.tile_state[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ready = __all(st != 0);
      // give up after kSpinLimit polls, or as soon as another tile has given up (a stalled
      // predecessor would otherwise make every later tile spin its full limit in turn)
      if (!ready && (++polls > kSpinLimit ||
                     ((polls & 1023u) == 0 &&
                      __hip_atomic_load(p.error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0))) {   // never taken in a correct run
        if (lane == 0) __hip_atomic_store(p.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (st == 0) st = kFlagPrefix;
        ready = true;
      }
    } while (!ready);
    const uint64_t has_prefix = __ballot((st & kFlagPrefix) != 0);
    const int stop = has_prefix ? __ffsll(static_cast<long long>(has_prefix)) - 1 : cs::kWave;
    exclusive += wave_sum(lane <= stop ? static_cast<uint32_t>(st) : 0u);
    if (has_prefix) break;
    first -= cs::kWave;
  }
  if (lane == 0)
    __hip_atomic_store(&p.tile_state[tile], kFlagPrefix | (exclusive + aggregate), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
  return exclusive;
}

// MODE kFused: the whole call in one launch (pass 1, look-back, pass 2), for the batches a serving
// step really has.  MODE kScoreOnly / kEmitOnly: pass 1 and pass 2 as launches of their own with a
// small scan of the per-wave totals between them, for batches of many thousand streams: there the
// one-launch form serialises (every tile takes a ticket from one address, about 16 ns each, and
// all tiles reach the look-back together, so the memory system idles while the prefixes resolve),
// and tiles need no order at all when the prefix comes from a scan.
constexpr int kFused = 0, kScoreOnly = 1, kEmitOnly = 2;

template <int G, bool PK, int MODE>
__global__ __launch_bounds__(kWavesPerTile * cs::kWave) void score_compact_kernel(ScoreParams p) {
  __shared__ uint32_t s_ticket;
  __shared__ uint32_t s_total[kWavesPerTile];
  __shared__ uint32_t s_exclusive;
  __shared__ uint64_t s_mask[MODE == kFused ? kWavesPerTile : 1][kMaskWords];
  const int lane = threadIdx.x & (cs::kWave - 1);
  const int wave = threadIdx.x / cs::kWave;
  if constexpr (MODE == kFused) {
    if (threadIdx.x == 0) {
      if (p.single_tile) {
        s_ticket = 0;
        *p.error = 0;                    // the word callers may inspect; nothing else of the workspace is used
      } else {
        s_ticket = atomicAdd(p.ticket, 1u);
      }
    }
    __syncthreads();
  }
  const uint32_t tile = MODE == kFused ? s_ticket : blockIdx.x;
  uint64_t* my_masks = s_mask[MODE == kFused ? wave : 0];
  const int s_begin = (static_cast<int>(tile) * kWavesPerTile + wave) * p.streams_per_wave;
  const int s_end = min(p.n_streams, s_begin + p.streams_per_wave);
  // The wave's frame ranges and frame types are fetched lane-parallel up front, so that the walk
  // over its streams does not pay a dependent memory round trip per stream for them.
  const int n_mine = max(0, s_end - s_begin);                       // <= 63 streams
  const int cu_l = lane <= n_mine && n_mine > 0 ? p.cu_frames[s_begin + lane] : 0;
  const int f_first = __builtin_amdgcn_readlane(cu_l, 0);
  const int f_stop = __builtin_amdgcn_readlane(cu_l, n_mine);
  const int ft_l = f_first + lane < f_stop ? p.frame_type[f_first + lane] : 0;
  auto frame_is_i = [&](int f) -> bool {
    const int rel = f - f_first;
    const int t = rel < cs::kWave ? __builtin_amdgcn_readlane(ft_l, rel) : static_cast<int>(p.frame_type[f]);
    return t == CS_FRAME_I;
  };
  uint32_t total = 0;
  int mask_words = MODE == kFused ? 0 : kMaskWords;               // only the one-launch form keeps ballot words in LDS
  // ---- pass 1, software pipelined over the wave's sweeps (stream by stream, frame by frame, 256
  //      token locations at a time): the loads of the next sweep are issued before the current one
  //      is scored, so two sweeps' worth of loads are in flight per wave.  The accumulated state of
  //      the next sweep comes from memory unless it is the same locations of the same stream one
  //      frame later; then it is what this sweep leaves in registers.
  auto first_sweep = [&](int i0) -> Sweep {
    Sweep w{i0, 0, 0, 0, false};
    while (w.i < n_mine) {                                         // skip streams without frames
      const int f0 = __builtin_amdgcn_readlane(cu_l, w.i), f1 = __builtin_amdgcn_readlane(cu_l, w.i + 1);
      if (f0 < f1) { w.s = s_begin + w.i; w.f = f0; w.t0 = 0; w.is_i = frame_is_i(f0); return w; }
      ++w.i;
    }
    return w;
  };
  auto next_sweep = [&](const Sweep& c) -> Sweep {
    Sweep w = c;
    if (c.t0 + kSweep < p.n_tok) { w.t0 = c.t0 + kSweep; return w; }
    const int f1 = __builtin_amdgcn_readlane(cu_l, c.i + 1);
    if (c.f + 1 < f1) { w.f = c.f + 1; w.t0 = 0; w.is_i = frame_is_i(w.f); return w; }
    return first_sweep(c.i + 1);
  };
  if constexpr (MODE != kEmitOnly) {
    Sweep cur = first_sweep(0);
    SweepRegs<G> rc, rn;
    if (cur.i < n_mine) {
      load_inputs<G, PK>(p, cur, lane, rc);
      load_acc<G, PK>(p, cur, lane, rc);
    }
    while (cur.i < n_mine) {
      const Sweep nxt = next_sweep(cur);
      const bool more = nxt.i < n_mine;
      const bool forward = more && nxt.s == cur.s && nxt.t0 == cur.t0;   // same locations, next frame
      if (more) {
        load_inputs<G, PK>(p, nxt, lane, rn);
        if (!forward) load_acc<G, PK>(p, nxt, lane, rn);
      }
      total += score_sweep<G, PK>(p, cur, lane, rc, my_masks, mask_words);
      if (forward) {
#pragma unroll
        for (int k = 0; k < kGroupsPerSweep; ++k)
#pragma unroll
          for (int q = 0; q < G * G; ++q) rn.acw[k][q] = rc.acw[k][q];
      }
      rc = rn;
      cur = nxt;
    }
  }
  const int64_t gw = static_cast<int64_t>(tile) * kWavesPerTile + wave;
  if constexpr (MODE == kScoreOnly) {
    if (lane == 0) { p.wave_total[gw] = total; s_total[wave] = total; }
    __syncthreads();
    if (threadIdx.x == 0) {
      uint32_t sum = 0;
#pragma unroll
      for (int w = 0; w < kWavesPerTile; ++w) sum += s_total[w];
      p.wg_total[tile] = sum;
    }
    return;
  }
  uint32_t base;
  if constexpr (MODE == kFused) {
    if (lane == 0) s_total[wave] = total;
    __syncthreads();
    if (wave == 0) {
      uint32_t aggregate = 0;
#pragma unroll
      for (int w = 0; w < kWavesPerTile; ++w) aggregate += s_total[w];
      const uint32_t exclusive = p.single_tile ? 0u : look_back(p, tile, aggregate, lane);
      if (lane == 0) s_exclusive = exclusive;
    }
    __syncthreads();
    base = s_exclusive;
    for (int w = 0; w < wave; ++w) base += s_total[w];
    mask_words = 0;
  } else {
    base = p.wg_total[tile];                                         // exclusive prefix by now
    for (int w = 0; w < wave; ++w) base += p.wave_total[gw - wave + w];
  }
  if constexpr (MODE == kEmitOnly && PK) {
    // The frames of a wave's streams are one contiguous run of keep bytes.  Taken a sweep at a time
    // the pass is a chain of dependent round trips (one 4-byte load per lane in flight); here the
    // keep words of kEmitAhead sweeps are requested before the first of them is ranked.
    const int spf = (p.n_tok + kSweep - 1) / kSweep;                 // sweeps per frame
    const int n_sw = (f_stop - f_first) * spf;
    auto keep_word = [&](int f, int t0) -> uint32_t {
      const int t = t0 + 4 * lane;
      return t < p.n_tok ? *reinterpret_cast<const uint32_t*>(p.keep + static_cast<size_t>(f) * p.n_tok + t) : 0u;
    };
    int pf = f_first, pt = 0;                                         // next sweep to request
    int f = f_first, t0 = 0;                                          // next sweep to rank
    uint32_t ring[kEmitAhead];
#pragma unroll
    for (int d = 0; d < kEmitAhead; ++d) {
      ring[d] = d < n_sw ? keep_word(pf, pt) : 0u;
      pt += kSweep;
      if (pt >= p.n_tok) { pt = 0; ++pf; }
    }
    for (int q = 0; q < n_sw; q += kEmitAhead) {
      uint32_t cur[kEmitAhead];
#pragma unroll
      for (int d = 0; d < kEmitAhead; ++d) cur[d] = ring[d];
#pragma unroll
      for (int d = 0; d < kEmitAhead; ++d) {
        ring[d] = q + kEmitAhead + d < n_sw ? keep_word(pf, pt) : 0u;
        pt += kSweep;
        if (pt >= p.n_tok) { pt = 0; ++pf; }
      }
#pragma unroll
      for (int d = 0; d < kEmitAhead; ++d) {
        if (q + d < n_sw) {
          if (t0 == 0 && lane == 0) p.kept_off[f] = static_cast<int32_t>(base);
          uint64_t mask[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) mask[k] = __ballot(((cur[d] >> (8 * k)) & 0xffu) != 0);
          uint32_t rank = 0, total = 0;
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            rank += lanes_below(mask[k]);
            total += __popcll(mask[k]);
          }
          const int32_t id = f * p.n_tok + t0 + 4 * lane;
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            if ((mask[k] >> lane) & 1) {
              p.kept_idx[base + rank] = id + k;
              ++rank;
            }
          }
          base += total;
          t0 += kSweep;
          if (t0 >= p.n_tok) { t0 = 0; ++f; }
        }
      }
    }
    if (s_end == p.n_streams && n_mine > 0 && lane == 0) p.kept_off[p.n_frames] = static_cast<int32_t>(base);
    return;
  }
  for (int i = 0; i < n_mine; ++i) {
    const int f0 = __builtin_amdgcn_readlane(cu_l, i), f1 = __builtin_amdgcn_readlane(cu_l, i + 1);
    for (int f = f0; f < f1; ++f) {
      if (lane == 0) p.kept_off[f] = static_cast<int32_t>(base);
      base += emit_frame<PK>(p, f, base, lane, my_masks, mask_words);
    }
    if (s_begin + i == p.n_streams - 1 && lane == 0) p.kept_off[p.n_frames] = static_cast<int32_t>(base);
  }
}

// Exclusive prefix of the per-workgroup totals, in place (one workgroup; 8 consecutive entries
// per thread and round).  Also clears the first workspace word (ticket and error flag), which
// this form does not otherwise use.
constexpr int kScanThreads = 1024, kScanPerThread = 8;

__global__ __launch_bounds__(kScanThreads) void scan_totals_kernel(uint64_t* first_word, uint32_t* totals, int64_t n) {
  __shared__ uint32_t s_part[kScanThreads / cs::kWave];
  __shared__ uint32_t s_run;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { s_run = 0; *first_word = 0; }
  __syncthreads();
  for (int64_t i0 = 0; i0 < n; i0 += kScanThreads * kScanPerThread) {
    const int64_t first = i0 + static_cast<int64_t>(tid) * kScanPerThread;
    uint32_t v[kScanPerThread], sum = 0;
#pragma unroll
    for (int u = 0; u < kScanPerThread; ++u) {
      v[u] = first + u < n ? totals[first + u] : 0u;
      sum += v[u];
    }
    uint32_t incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t t = __shfl_up(incl, off);
      if (lane >= off) incl += t;
    }
    if (lane == 63) s_part[wave] = incl;
    __syncthreads();
    uint32_t run = s_run + incl - sum;
    for (int w = 0; w < wave; ++w) run += s_part[w];
#pragma unroll
    for (int u = 0; u < kScanPerThread; ++u) {
      if (first + u < n) totals[first + u] = run;
      run += v[u];
    }
    __syncthreads();
    if (tid == kScanThreads - 1) s_run = run;
    __syncthreads();
  }
}

// Above this many streams the call is three launches (see score_compact_kernel).
constexpr int kFusedMaxStreams = 4096;

struct SplitPlan {
  int streams_per_wave;
  int64_t n_waves, n_wgs;
};

inline SplitPlan split_plan(int n_streams) {
  SplitPlan s;
  int k = (n_streams + 32767) / 32768;                    // a few sweeps per wave, tens of thousands of waves
  s.streams_per_wave = k < 1 ? 1 : (k > 63 ? 63 : k);
  s.n_waves = (static_cast<int64_t>(n_streams) + s.streams_per_wave - 1) / s.streams_per_wave;
  s.n_wgs = (s.n_waves + kWavesPerTile - 1) / kWavesPerTile;
  return s;
}

// Streams per wave: one for the batches a serving step really has (all the parallelism there is);
// for very large batches a wave sweeps several consecutive streams so that a tile carries enough
// work to amortise its look-back and the number of tiles stays in the low thousands.
inline int streams_per_wave_for(int n_streams) {
  int k = (n_streams + 8191) / 8192;
  return k < 1 ? 1 : (k > 63 ? 63 : k);     // 63: a wave fetches its streams' frame ranges in one load
}

inline int tiles_for(int n_streams) {
  const int per_tile = kWavesPerTile * streams_per_wave_for(n_streams);
  return (n_streams + per_tile - 1) / per_tile;
}

}  // namespace

extern "C" size_t cs_score_compact_workspace(int32_t n_streams, int32_t n_frames, int32_t grid_h,
                                             int32_t grid_w, int32_t group) {
  (void)n_frames; (void)grid_h; (void)grid_w; (void)group;
  if (n_streams < 0) return 0;
  if (n_streams > kFusedMaxStreams)
    return 8 + ((static_cast<size_t>(split_plan(n_streams).n_wgs) * (kWavesPerTile + 1) * sizeof(uint32_t) + 7) & ~size_t(7));
  return (static_cast<size_t>(tiles_for(n_streams)) + 1) * sizeof(uint64_t);
}

// Scratch of the entry point that allocates nothing (cs_score_compact_noalloc): the look-back words
// of the one-launch form for up to 4,096 streams ((1,024 tiles + 1) x 8 bytes).  Every GPU the
// library runs on holds its own copy, at its own address, until the process ends; host code reaches
// it only through the pointer hipGetSymbolAddress returns for the current device.
constexpr size_t kNoAllocScratchBytes = 8448;
static __device__ __align__(256) unsigned char g_score_scratch[kNoAllocScratchBytes];

namespace {

int score_compact_call(const int16_t* mv, const uint32_t* sad, const uint8_t* intra,
                       const uint8_t* frame_type, const int32_t* cu_frames,
                       uint8_t* acc_mask, int32_t n_streams, int32_t n_frames,
                       int32_t grid_h, int32_t grid_w, int32_t group,
                       uint32_t tau_mv_sq, uint32_t tau_sad, int32_t use_residual,
                       uint8_t* keep_mask, int32_t* kept_idx, int32_t* kept_off,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (n_streams < 0 || n_frames < 0 || grid_h < 1 || grid_w < 1 || group < 1) return CS_EINVAL;
  if (group != 1 && group != 2) return CS_EUNSUPPORTED;
  if (grid_h % group || grid_w % group) return CS_EINVAL;
  if (!kept_off) return CS_EINVAL;
  if ((use_residual != 0) != (sad != nullptr)) return CS_EINVAL;
  const int64_t n_tok = static_cast<int64_t>(grid_h / group) * (grid_w / group);
  const int64_t n_patch = static_cast<int64_t>(grid_h) * grid_w;
  if (n_tok * n_frames >= (1ll << 31) || n_patch * n_frames >= (1ll << 31)) return CS_EUNSUPPORTED;
  hipStream_t st = cs::as_stream(stream);
  if (n_streams == 0 || n_frames == 0) {
    const int n = n_frames + 1;
    hipLaunchKernelGGL(zero_offsets_kernel, dim3((n + 255) / 256), dim3(256), 0, st, kept_off, n);
    return cs::note_hip(hipGetLastError());
  }
  if (!mv || !frame_type || !cu_frames || !keep_mask || !kept_idx) return CS_EINVAL;
  const size_t need = cs_score_compact_workspace(n_streams, n_frames, grid_h, grid_w, group);
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 7u))
    return CS_EWORKSPACE;

  const bool split = n_streams > kFusedMaxStreams;
  const SplitPlan sp = split_plan(n_streams);
  if (split && sp.n_wgs >= (1ll << 31)) return CS_EUNSUPPORTED;
  const int n_tiles = split ? static_cast<int>(sp.n_wgs) : tiles_for(n_streams);
  ScoreParams p;
  p.mv = reinterpret_cast<const uint32_t*>(mv);
  p.sad = sad;
  p.intra = intra;
  p.frame_type = frame_type;
  p.cu_frames = cu_frames;
  p.acc = acc_mask;
  p.keep = keep_mask;
  p.kept_idx = kept_idx;
  p.kept_off = kept_off;
  p.ticket = reinterpret_cast<uint32_t*>(workspace);
  p.error = p.ticket + 1;
  p.tile_state = reinterpret_cast<uint64_t*>(workspace) + 1;
  p.wg_total = reinterpret_cast<uint32_t*>(workspace) + 2;
  p.wave_total = p.wg_total + sp.n_wgs;
  p.n_streams = n_streams;
  p.n_frames = n_frames;
  p.grid_w = grid_w;
  p.tok_w = grid_w / group;
  p.n_patch = static_cast<int32_t>(n_patch);
  p.n_tok = static_cast<int32_t>(n_tok);
  p.tau_mv_sq = tau_mv_sq;
  p.tau_sad = tau_sad;
  p.use_residual = use_residual ? 1 : 0;
  p.streams_per_wave = split ? sp.streams_per_wave : streams_per_wave_for(n_streams);

  p.single_tile = !split && n_tiles == 1 ? 1 : 0;
  if (!split && n_tiles > 1) {                              // ticket + error word, tile states
    const int n_words = n_tiles + 1;
    hipLaunchKernelGGL(clear_words_kernel, dim3((n_words + 255) / 256), dim3(256), 0, st,
                       reinterpret_cast<uint64_t*>(workspace), n_words);
  }
  const dim3 grid(n_tiles), block(kWavesPerTile * cs::kWave);
  // packed accesses need 16-byte aligned metadata rows and 4-byte aligned byte rows
  const bool packed = group == 1 && n_patch % 4 == 0 && cs::aligned16(mv) && (!sad || cs::aligned16(sad)) &&
                      !(reinterpret_cast<uintptr_t>(intra) & 3u) && !(reinterpret_cast<uintptr_t>(acc_mask) & 3u) &&
                      !(reinterpret_cast<uintptr_t>(keep_mask) & 3u);
#define CS_LAUNCH_SCORE(MODE)                                                                        \
  do {                                                                                               \
    if (packed)                                                                                      \
      hipLaunchKernelGGL((score_compact_kernel<1, true, MODE>), grid, block, 0, st, p);              \
    else if (group == 1)                                                                             \
      hipLaunchKernelGGL((score_compact_kernel<1, false, MODE>), grid, block, 0, st, p);             \
    else                                                                                             \
      hipLaunchKernelGGL((score_compact_kernel<2, false, MODE>), grid, block, 0, st, p);             \
  } while (0)
  if (!split) {
    CS_LAUNCH_SCORE(kFused);
  } else {
    CS_LAUNCH_SCORE(kScoreOnly);
    hipLaunchKernelGGL(scan_totals_kernel, dim3(1), dim3(kScanThreads), 0, st,
                       reinterpret_cast<uint64_t*>(workspace), p.wg_total, sp.n_wgs);
    CS_LAUNCH_SCORE(kEmitOnly);
  }
#undef CS_LAUNCH_SCORE
  return cs::note_hip(hipGetLastError());
}

// The entry point that allocates nothing serves up to kNoAllocMaxStreams streams.
constexpr int kNoAllocMaxStreams = kFusedMaxStreams;
static_assert((kFusedMaxStreams / kWavesPerTile + 1) * sizeof(uint64_t) <= kNoAllocScratchBytes, "scratch too small");

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of the scratch array on the current device (resolved once per device).
int score_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return cs::note_hip(e);
  if (dev < 0 || dev >= kMaxDevices) return CS_EUNSUPPORTED;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_score_scratch));
    if (e != hipSuccess || !ptr) return cs::note_hip(e == hipSuccess ? hipErrorInvalidSymbol : e);
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CS_OK;
}

}  // namespace

extern "C" int cs_score_compact(const int16_t* mv, const uint32_t* sad, const uint8_t* intra,
                                const uint8_t* frame_type, const int32_t* cu_frames,
                                uint8_t* acc_mask, int32_t n_streams, int32_t n_frames,
                                int32_t grid_h, int32_t grid_w, int32_t group,
                                uint32_t tau_mv_sq, uint32_t tau_sad, int32_t use_residual,
                                uint8_t* keep_mask, int32_t* kept_idx, int32_t* kept_off,
                                void* workspace, size_t workspace_bytes, void* stream) {
  return score_compact_call(mv, sad, intra, frame_type, cu_frames, acc_mask, n_streams, n_frames, grid_h, grid_w,
                            group, tau_mv_sq, tau_sad, use_residual, keep_mask, kept_idx, kept_off, workspace,
                            workspace_bytes, stream);
}

extern "C" int cs_score_compact_noalloc(const int16_t* mv, const uint32_t* sad, const uint8_t* intra,
                                        const uint8_t* frame_type, const int32_t* cu_frames,
                                        uint8_t* acc_mask, int32_t n_streams, int32_t n_frames,
                                        int32_t grid_h, int32_t grid_w, int32_t group,
                                        uint32_t tau_mv_sq, uint32_t tau_sad, int32_t use_residual,
                                        uint8_t* keep_mask, int32_t* kept_idx, int32_t* kept_off,
                                        void* stream) {
  if (n_streams > kNoAllocMaxStreams) return CS_EUNSUPPORTED;      // beyond the static scratch
  void* scratch = nullptr;
  const int e = score_scratch(&scratch);
  if (e != CS_OK) return e;
  // the one-launch form clears the look-back words it uses with a kernel of its own on `stream`,
  // so the contents the previous call left in the scratch never matter
  return score_compact_call(mv, sad, intra, frame_type, cu_frames, acc_mask, n_streams, n_frames, grid_h, grid_w,
                            group, tau_mv_sq, tau_sad, use_residual, keep_mask, kept_idx, kept_off, scratch,
                            kNoAllocScratchBytes, stream);
}
