// Block-to-patch projection.  Paper Sec. 3.3.1 (paragraph on mapping codec changes to ViT
// patches): block rectangles are in source-frame pixels, patches in model-input pixels; the
// rectangles are rescaled and every patch gets the strongest motion (Eq. 1) among the blocks that
// land on it.  Sec. 3.3.2: a patch touched by an intra-coded block is flagged.
//
// One workgroup per frame.  The frame's patch table lives in LDS as 64-bit keys
//     key = |v|^2 << 32 | (dx + 32768) << 16 | (dy + 32768)
// so that "largest magnitude, ties to the lexicographically largest vector" is an unsigned
// maximum and the winning vector comes back out of the key: blocks are streamed once (one 16-byte
// load each), each computes its patch range with exact integer arithmetic and raises the keys of
// the patches it overlaps (ds_max_u64; a plain read first skips the atomic when the patch already
// holds at least as much, which is the common case inside a moving region).  The order in which
// blocks arrive cannot change the result.  Divisions by the two launch constants
// patch * src_w and patch * src_h are multiplications by a precomputed reciprocal that is exact for
// the numerators that can occur (below 2^29).
#include "common.h"

namespace {

constexpr int kProjectThreads = 1024;
constexpr int kBatch = 4;
constexpr int kNumeratorBits = 29;

struct ExactDiv {                // q = (n * mul) >> shift == n / d for every n < 2^kNumeratorBits
  uint32_t mul;
  uint32_t shift;
};

ExactDiv exact_div(uint32_t d) {
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;                                  // l = ceil(log2 d)
  const uint64_t two = 1ull << (kNumeratorBits + l);
  ExactDiv e;
  e.mul = static_cast<uint32_t>((two + d - 1) / d);             // < 2^(kNumeratorBits + 1)
  e.shift = kNumeratorBits + l;
  return e;
}

__device__ __forceinline__ uint32_t div_by(uint32_t n, ExactDiv e) {
  return static_cast<uint32_t>((static_cast<uint64_t>(n) * e.mul) >> e.shift);
}

struct ProjectParams {
  const cs::u32x4* __restrict__ blocks;
  const int32_t* __restrict__ cu_blocks;
  uint32_t* __restrict__ mv;         // [F][P] packed (dx, dy)
  uint8_t* __restrict__ intra;       // [F][P]
  uint32_t src_w, src_h, in_w, in_h;
  uint32_t den_x, den_y;             // patch * src_w, patch * src_h
  ExactDiv div_x, div_y;
  int32_t grid_h, grid_w, n_patch;
};

__global__ __launch_bounds__(kProjectThreads) void project_blocks_kernel(ProjectParams p) {
  extern __shared__ unsigned long long s_key[];                         // [n_patch]
  uint32_t* s_intra = reinterpret_cast<uint32_t*>(s_key + p.n_patch);  // bitmap, n_patch bits
  const int tid = threadIdx.x;
  const int frame = blockIdx.x;
  for (int i = tid; i < p.n_patch; i += kProjectThreads) s_key[i] = 0ull;
  for (int i = tid; i < (p.n_patch + 31) / 32; i += kProjectThreads) s_intra[i] = 0u;
  __syncthreads();

  const int begin = p.cu_blocks[frame], end = p.cu_blocks[frame + 1];
  auto apply = [&](const cs::u32x4 rec) {
    const uint32_t x = rec.x & 0xffffu, y = rec.x >> 16, w = rec.y & 0xffffu, h = rec.y >> 16;
    const int dx = static_cast<int16_t>(rec.z & 0xffffu), dy = static_cast<int16_t>(rec.z >> 16);
    const bool is_intra = (rec.w & 1u) != 0;
    const uint32_t mag = static_cast<uint32_t>(dx * dx) + static_cast<uint32_t>(dy * dy);   // up to 2^31
    if (!is_intra && mag == 0u) return;                       // a zero vector changes no patch
    // footprint clipped to the frame; nothing left -> no footprint
    const uint32_t lo_x = min(x, p.src_w), hi_x = min(x + w, p.src_w);
    const uint32_t lo_y = min(y, p.src_h), hi_y = min(y + h, p.src_h);
    if (hi_x <= lo_x || hi_y <= lo_y) return;
    // patch columns c with lo*in < (c+1)*den and hi*in > c*den (positive overlap), same for rows
    const int c0 = static_cast<int>(div_by(lo_x * p.in_w, p.div_x));
    const int c1 = min(static_cast<int>(div_by(hi_x * p.in_w + p.den_x - 1u, p.div_x)) - 1, p.grid_w - 1);
    const int r0 = static_cast<int>(div_by(lo_y * p.in_h, p.div_y));
    const int r1 = min(static_cast<int>(div_by(hi_y * p.in_h + p.den_y - 1u, p.div_y)) - 1, p.grid_h - 1);
    const unsigned long long key = (static_cast<unsigned long long>(mag) << 32) |
                                   (static_cast<uint32_t>(dx + 32768) << 16) | static_cast<uint32_t>(dy + 32768);
    for (int r = r0; r <= r1; ++r)
      for (int c = c0; c <= c1; ++c) {
        const int cell = r * p.grid_w + c;
        if (is_intra) {
          const uint32_t bit = 1u << (cell & 31);
          if (!(s_intra[cell >> 5] & bit)) atomicOr(&s_intra[cell >> 5], bit);
        } else if (s_key[cell] < key) {
          atomicMax(&s_key[cell], key);
        }
      }
  };
  // kBatch records in flight per thread (a record past the end is replaced by an empty one)
  for (int i0 = begin + tid; i0 < end; i0 += kProjectThreads * kBatch) {
    cs::u32x4 rec[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int i = i0 + u * kProjectThreads;
      rec[u] = i < end ? __builtin_nontemporal_load(p.blocks + i) : cs::u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) apply(rec[u]);
  }
  __syncthreads();

  uint32_t* mv = p.mv + static_cast<int64_t>(frame) * p.n_patch;
  uint8_t* intra = p.intra + static_cast<int64_t>(frame) * p.n_patch;
  for (int i = tid; i < p.n_patch; i += kProjectThreads) {
    const unsigned long long key = s_key[i];                  // 0: no moving inter block here
    const uint32_t low = static_cast<uint32_t>(key);
    const uint32_t dx16 = key == 0ull ? 0u : ((low >> 16) - 32768u) & 0xffffu;
    const uint32_t dy16 = key == 0ull ? 0u : ((low & 0xffffu) - 32768u) & 0xffffu;
    mv[i] = dx16 | (dy16 << 16);
    intra[i] = (s_intra[i >> 5] >> (i & 31)) & 1u;
  }
}

}  // namespace

extern "C" int cs_project_blocks(const cs_block* blocks, const int32_t* cu_blocks, int32_t n_frames,
                                 int32_t src_w, int32_t src_h, int32_t in_w, int32_t in_h,
                                 int32_t patch, int32_t grid_h, int32_t grid_w, int16_t* mv,
                                 uint8_t* intra, void* stream) {
  static_assert(sizeof(cs_block) == 16, "block records are 16 bytes");
  if (n_frames < 0 || src_w < 1 || src_h < 1 || in_w < 1 || in_h < 1 || patch < 1 || grid_h < 1 || grid_w < 1)
    return CS_EINVAL;
  if (n_frames == 0) return CS_OK;
  if (!blocks || !cu_blocks || !mv || !intra) return CS_EINVAL;
  if (src_w > 16384 || src_h > 16384 || in_w > 16384 || in_h > 16384 || patch > 1024) return CS_EUNSUPPORTED;
  const int64_t n_patch = static_cast<int64_t>(grid_h) * grid_w;
  if (n_patch > 7168) return CS_EUNSUPPORTED;       // the frame's patch table stays in LDS (under 64 KB)
  if (!cs::aligned16(blocks) || (reinterpret_cast<uintptr_t>(mv) & 3u)) return CS_EUNSUPPORTED;

  ProjectParams p;
  p.blocks = reinterpret_cast<const cs::u32x4*>(blocks);
  p.cu_blocks = cu_blocks;
  p.mv = reinterpret_cast<uint32_t*>(mv);
  p.intra = intra;
  p.src_w = src_w; p.src_h = src_h; p.in_w = in_w; p.in_h = in_h;
  p.den_x = static_cast<uint32_t>(patch) * src_w;
  p.den_y = static_cast<uint32_t>(patch) * src_h;
  p.div_x = exact_div(p.den_x);
  p.div_y = exact_div(p.den_y);
  p.grid_h = grid_h; p.grid_w = grid_w;
  p.n_patch = static_cast<int32_t>(n_patch);
  const size_t lds = static_cast<size_t>(n_patch) * 8 + static_cast<size_t>((n_patch + 31) / 32) * 4;
  hipLaunchKernelGGL(project_blocks_kernel, dim3(static_cast<unsigned>(n_frames)), dim3(kProjectThreads),
                     lds, cs::as_stream(stream), p);
  return cs::note_hip(hipGetLastError());
}
