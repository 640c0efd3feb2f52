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
#include "common.h"

namespace {

constexpr int kWavesPerTile = 4;
constexpr int kGroupsPerSweep = 4;                       // 64-token groups per lane sweep
constexpr int kSweep = cs::kWave * kGroupsPerSweep;      // token locations per sweep
constexpr uint64_t kFlagAggregate = 1ull << 62;
constexpr uint64_t kFlagPrefix = 1ull << 63;
constexpr uint32_t kSpinLimit = 1u << 24;
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
  uint64_t* tile_state;                  // workspace + 8
  int32_t n_streams, n_frames, grid_w, tok_w, n_patch, n_tok;
  int32_t streams_per_wave;              // consecutive streams swept by one wave (1 for small batches)
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

// Scores one frame of one stream; returns the number of kept tokens (wave-uniform).
template <int G>
__device__ uint32_t score_frame(const ScoreParams& p, int s, int f, bool is_i, int lane,
                                uint64_t* mask_cache, int& mask_words) {
  constexpr int Q = G * G;
  const size_t pbase = static_cast<size_t>(f) * p.n_patch;
  uint8_t* __restrict__ keep = p.keep + static_cast<size_t>(f) * p.n_tok;
  uint8_t* __restrict__ acc = p.acc ? p.acc + static_cast<size_t>(s) * p.n_patch : nullptr;
  uint32_t count = 0;
  for (int t0 = 0; t0 < p.n_tok; t0 += kSweep) {
    bool bit[kGroupsPerSweep];
    if (is_i) {
      // an I-frame keeps everything, resets the accumulation and its metadata is not read
#pragma unroll
      for (int k = 0; k < kGroupsPerSweep; ++k) {
        const int t = t0 + k * cs::kWave + lane;
        bit[k] = t < p.n_tok;
        if (bit[k]) {
          keep[t] = 1;
          if (acc) {
#pragma unroll
            for (int q = 0; q < Q; ++q) acc[patch_of<G>(p, t, q / G, q % G)] = 0;
          }
        }
      }
    } else {
      uint32_t mvw[kGroupsPerSweep][Q], sdw[kGroupsPerSweep][Q];
      uint8_t inw[kGroupsPerSweep][Q], acw[kGroupsPerSweep][Q];
      int pidx[kGroupsPerSweep][Q];
      // all loads of the sweep first, so that they are in flight together
#pragma unroll
      for (int k = 0; k < kGroupsPerSweep; ++k) {
        const int t = t0 + k * cs::kWave + lane;
        const bool valid = t < p.n_tok;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
          const int pi = valid ? patch_of<G>(p, t, q / G, q % G) : 0;
          pidx[k][q] = pi;
          mvw[k][q] = valid ? p.mv[pbase + pi] : 0u;
          sdw[k][q] = (valid && p.use_residual) ? p.sad[pbase + pi] : 0u;
          inw[k][q] = (valid && p.intra) ? p.intra[pbase + pi] : uint8_t(0);
          acw[k][q] = (valid && acc) ? acc[pi] : uint8_t(0);
        }
      }
#pragma unroll
      for (int k = 0; k < kGroupsPerSweep; ++k) {
        const int t = t0 + k * cs::kWave + lane;
        const bool valid = t < p.n_tok;
        bool any = false;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
          const int dx = static_cast<int16_t>(mvw[k][q] & 0xffffu);
          const int dy = static_cast<int16_t>(mvw[k][q] >> 16);
          const uint32_t m = static_cast<uint32_t>(dx * dx) + static_cast<uint32_t>(dy * dy);
          const bool d_mv = m >= p.tau_mv_sq;                                        // Eq. 3
          const bool d_res = p.use_residual && !d_mv && sdw[k][q] >= p.tau_sad;     // Eq. 4
          const bool d = d_mv || d_res || inw[k][q] != 0;                            // Eq. 5
          bool sel = d;
          if (acc) {
            sel = d || acw[k][q] != 0;                     // selected now or earlier in this GOP
            if (valid && sel && acw[k][q] == 0) acc[pidx[k][q]] = 1;
          }
          any = any || sel;
        }
        bit[k] = valid && any;
        if (valid) keep[t] = any ? 1 : 0;
      }
    }
#pragma unroll
    for (int k = 0; k < kGroupsPerSweep; ++k) {
      const uint64_t mask = __ballot(bit[k]);
      if (mask_words < kMaskWords && lane == 0) mask_cache[mask_words] = mask;   // for pass 2
      ++mask_words;
      count += __popcll(mask);
    }
  }
  return count;
}

// Writes the dense ids of the kept tokens of frame f starting at kept_idx[base]; returns count.
// The ballot words of pass 1 come back from LDS while they fit there (no memory round trip in
// this pass); beyond that the wave re-reads its own keep bytes.
__device__ uint32_t emit_frame(const ScoreParams& p, int f, uint32_t base, int lane,
                               const uint64_t* mask_cache, int& mask_words) {
  const uint8_t* keep = p.keep + static_cast<size_t>(f) * p.n_tok;
  const int32_t id0 = f * p.n_tok;
  uint32_t count = 0;
  for (int t0 = 0; t0 < p.n_tok; t0 += kSweep) {
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
      if (!ready && ++polls > kSpinLimit) {               // never taken in a correct run
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

template <int G>
__global__ __launch_bounds__(kWavesPerTile * cs::kWave) void score_compact_kernel(ScoreParams p) {
  __shared__ uint32_t s_ticket;
  __shared__ uint32_t s_total[kWavesPerTile];
  __shared__ uint32_t s_exclusive;
  __shared__ uint64_t s_mask[kWavesPerTile][kMaskWords];
  const int lane = threadIdx.x & (cs::kWave - 1);
  const int wave = threadIdx.x / cs::kWave;
  if (threadIdx.x == 0) s_ticket = atomicAdd(p.ticket, 1u);
  __syncthreads();
  const uint32_t tile = s_ticket;
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
  int mask_words = 0;
  for (int i = 0; i < n_mine; ++i) {
    const int f0 = __builtin_amdgcn_readlane(cu_l, i), f1 = __builtin_amdgcn_readlane(cu_l, i + 1);
    for (int f = f0; f < f1; ++f)
      total += score_frame<G>(p, s_begin + i, f, frame_is_i(f), lane, s_mask[wave], mask_words);
  }
  if (lane == 0) s_total[wave] = total;
  __syncthreads();
  if (wave == 0) {
    uint32_t aggregate = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerTile; ++w) aggregate += s_total[w];
    const uint32_t exclusive = look_back(p, tile, aggregate, lane);
    if (lane == 0) s_exclusive = exclusive;
  }
  __syncthreads();
  uint32_t base = s_exclusive;
  for (int w = 0; w < wave; ++w) base += s_total[w];
  mask_words = 0;
  for (int i = 0; i < n_mine; ++i) {
    const int f0 = __builtin_amdgcn_readlane(cu_l, i), f1 = __builtin_amdgcn_readlane(cu_l, i + 1);
    for (int f = f0; f < f1; ++f) {
      if (lane == 0) p.kept_off[f] = static_cast<int32_t>(base);
      base += emit_frame(p, f, base, lane, s_mask[wave], mask_words);
    }
    if (s_begin + i == p.n_streams - 1 && lane == 0) p.kept_off[p.n_frames] = static_cast<int32_t>(base);
  }
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
  return (static_cast<size_t>(tiles_for(n_streams)) + 1) * sizeof(uint64_t);
}

extern "C" int cs_score_compact(const int16_t* mv, const uint32_t* sad, const uint8_t* intra,
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

  const int n_tiles = tiles_for(n_streams);
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
  p.n_streams = n_streams;
  p.n_frames = n_frames;
  p.grid_w = grid_w;
  p.tok_w = grid_w / group;
  p.n_patch = static_cast<int32_t>(n_patch);
  p.n_tok = static_cast<int32_t>(n_tok);
  p.tau_mv_sq = tau_mv_sq;
  p.tau_sad = tau_sad;
  p.use_residual = use_residual ? 1 : 0;
  p.streams_per_wave = streams_per_wave_for(n_streams);

  const int n_words = n_tiles + 1;
  hipLaunchKernelGGL(clear_words_kernel, dim3((n_words + 255) / 256), dim3(256), 0, st,
                     reinterpret_cast<uint64_t*>(workspace), n_words);
  const dim3 grid(n_tiles), block(kWavesPerTile * cs::kWave);
  if (group == 1)
    hipLaunchKernelGGL(score_compact_kernel<1>, grid, block, 0, st, p);
  else
    hipLaunchKernelGGL(score_compact_kernel<2>, grid, block, 0, st, p);
  return cs::note_hip(hipGetLastError());
}
