// Residual proxy.  Paper Sec. 4 (Codec Processing): the decoder hands out no residuals, so they
// are approximated from pixels: the previous decoded frame is shifted by the motion vectors,
// compared with the current frame, and a patch is scored by the average absolute pixel difference
// inside it (the per-patch counterpart of the block residual of Eq. 2; input of the rescue rule, Eq. 4).
//
// Three launches on the caller's stream; the output array doubles as the accumulator:
//   1. clear the per-patch sums;
//   2. residual_sum_kernel: a workgroup owns a run of source rows inside one patch row of one
//      frame.  A thread owns a 4-pixel group of columns (consecutive lanes, consecutive groups:
//      every load of a wave is one contiguous span) and walks down the rows a cell row of the
//      motion field at a time: one vector, then for four pixel rows at once the current pixels
//      (one dword) and the reference pixels as two aligned dwords joined by a byte funnel shift
//      (per-pixel clamped byte loads only where the reference leaves the frame), twelve
//      independent loads in flight.  |a - b| over four pixels is one v_sad_u8; a group that
//      straddles a patch border is split by byte masks fixed per thread, so the row loop has no
//      patch arithmetic at all.  Sums go thread -> LDS (per patch column) -> one global atomic
//      per workgroup and patch;
//   3. residual_mean_kernel: sum -> floor(256 * sum / pixels of the patch).
// Integer adds commute, so the result is bit exact whatever the order.
#include "common.h"

namespace {

constexpr int kNumeratorBits = 29;

struct ExactDiv {                // q = (n * mul) >> shift == n / d for every n < 2^kNumeratorBits
  uint32_t mul;
  uint32_t shift;
};

ExactDiv exact_div(uint32_t d) {
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  const uint64_t two = 1ull << (kNumeratorBits + l);
  ExactDiv e;
  e.mul = static_cast<uint32_t>((two + d - 1) / d);
  e.shift = kNumeratorBits + l;
  return e;
}

__device__ __forceinline__ uint32_t div_by(uint32_t n, ExactDiv e) {
  return static_cast<uint32_t>((static_cast<uint64_t>(n) * e.mul) >> e.shift);
}

struct ResidualParams {
  const uint8_t* __restrict__ cur;
  const uint8_t* __restrict__ prev;
  const uint32_t* __restrict__ field;     // [F][cells_h][cells_w] packed (dx, dy), quarter pixels
  uint32_t* __restrict__ res;             // [F][P]: sums, then scores
  int64_t pitch, frame_stride;
  int32_t n_frames, src_w, src_h, cell_shift, cells_w, cells_h;
  uint32_t in_w, in_h, den_x, den_y;      // den = patch * src size
  ExactDiv div_x;
  int32_t grid_h, grid_w, n_sub;
};

// first source coordinate of patch index i along an axis: ceil(i * den / n_in), capped at n_src
__device__ __forceinline__ int first_coord(int i, uint32_t den, uint32_t n_in, int n_src) {
  const unsigned long long v = (static_cast<unsigned long long>(i) * den + n_in - 1) / n_in;
  return v < static_cast<unsigned long long>(n_src) ? static_cast<int>(v) : n_src;
}

__global__ __launch_bounds__(256) void clear_sums_kernel(uint32_t* p, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

__global__ __launch_bounds__(256) void residual_sum_kernel(ResidualParams p) {
  extern __shared__ uint32_t s_sum[];                       // [grid_w]
  const int tid = threadIdx.x;
  const int sub = blockIdx.x % p.n_sub;
  const int band = (blockIdx.x / p.n_sub) % p.grid_h;
  const int frame = blockIdx.x / (p.n_sub * p.grid_h);
  const int y_lo = first_coord(band, p.den_y, p.in_h, p.src_h);
  const int y_hi = first_coord(band + 1, p.den_y, p.in_h, p.src_h);
  if (y_lo >= y_hi) return;                                 // uniform for the workgroup
  // the band's rows in quads (rows 4q .. 4q+3, the unit of the row loop), dealt to its n_sub workgroups
  const int q_lo = y_lo >> 2, n_quads = ((y_hi - 1) >> 2) + 1 - q_lo;
  const int q_begin = q_lo + static_cast<int>(static_cast<int64_t>(n_quads) * sub / p.n_sub);
  const int q_end = q_lo + static_cast<int>(static_cast<int64_t>(n_quads) * (sub + 1) / p.n_sub);
  const int y_begin = max(y_lo, 4 * q_begin), y_end = min(y_hi, 4 * q_end);
  if (y_begin >= y_end) return;

  for (int i = tid; i < p.grid_w; i += 256) s_sum[i] = 0u;
  __syncthreads();

  const int W = p.src_w, H = p.src_h;
  const int groups = (W + 3) / 4;                                    // 4-pixel groups along a row
  const uint8_t* cur = p.cur + static_cast<int64_t>(frame) * p.frame_stride;
  const uint8_t* prev = p.prev + static_cast<int64_t>(frame) * p.frame_stride;
  const uint32_t* field = p.field + static_cast<int64_t>(frame) * p.cells_h * p.cells_w;
  const int cell = 1 << p.cell_shift;

  for (int k = tid; k < groups; k += 256) {
    // ---- the group's patch column(s) and the byte masks that split it between them
    const int x = 4 * k;
    int col_a = static_cast<int>(div_by(static_cast<uint32_t>(x) * p.in_w, p.div_x)), col_b = 0;
    uint32_t mask_a = 0u, mask_b = 0u;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (x + t < W) {
        const int c = static_cast<int>(div_by(static_cast<uint32_t>(x + t) * p.in_w, p.div_x));
        if (c == col_a) mask_a |= 0xffu << (8 * t);
        else { mask_b |= 0xffu << (8 * t); col_b = c; }     // columns are at least 4 pixels wide: one other column at most
      }
    }
    if (col_a >= p.grid_w) mask_a = 0u;
    if (col_b >= p.grid_w) mask_b = 0u;
    uint32_t acc_a = 0u, acc_b = 0u;
    // ---- down the rows, one cell row of the motion field at a time, four pixel rows per batch
    const int yc_last = (y_end - 1) >> p.cell_shift;
    const uint32_t* fcol = field + (x >> p.cell_shift);
    uint32_t mv_next = fcol[static_cast<int64_t>(y_begin >> p.cell_shift) * p.cells_w];
    for (int yc = y_begin >> p.cell_shift; yc <= yc_last; ++yc) {
      const uint32_t mv = mv_next;
      mv_next = fcol[static_cast<int64_t>(min(yc + 1, yc_last)) * p.cells_w];     // one cell row ahead
      const int ox = (static_cast<int>(static_cast<int16_t>(mv & 0xffffu)) + 2) >> 2;
      const int oy = (static_cast<int>(static_cast<int16_t>(mv >> 16)) + 2) >> 2;
      const int xs = x + ox;
      const bool fast = xs >= 0 && xs + 3 <= W - 1;         // the reference group lies inside the row
      const int a0 = fast ? (xs & ~3) : 0;                   // two aligned dwords, both inside the row
      const int a1 = fast && (xs & 3) ? a0 + 4 : a0;
      for (int r4 = 0; r4 < cell; r4 += 4) {
        uint32_t c4[4], lo[4], hi[4];
        bool live[4];
#pragma unroll
        for (int dy = 0; dy < 4; ++dy) {
          const int y = (yc << p.cell_shift) + r4 + dy;
          live[dy] = y >= y_begin && y < y_end;
          const int yv = min(max(y, y_begin), y_end - 1);    // a row of this workgroup in any case
          const int yy = min(max(yv + oy, 0), H - 1);
          const uint8_t* prow = prev + static_cast<int64_t>(yy) * p.pitch;
          c4[dy] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(cur + static_cast<int64_t>(yv) * p.pitch + x));
          lo[dy] = *reinterpret_cast<const uint32_t*>(prow + a0);
          hi[dy] = *reinterpret_cast<const uint32_t*>(prow + a1);
        }
#pragma unroll
        for (int dy = 0; dy < 4; ++dy) {
          uint32_t pred = __builtin_amdgcn_alignbyte(hi[dy], lo[dy], static_cast<uint32_t>(xs & 3));
          if (!fast) {                                       // reference leaves the frame: clamp per pixel
            const int y = (yc << p.cell_shift) + r4 + dy;
            const int yv = min(max(y, y_begin), y_end - 1);
            const uint8_t* prow = prev + static_cast<int64_t>(min(max(yv + oy, 0), H - 1)) * p.pitch;
            pred = 0u;
#pragma unroll
            for (int t = 0; t < 4; ++t) pred |= static_cast<uint32_t>(prow[min(max(xs + t, 0), W - 1)]) << (8 * t);
          }
          const uint32_t ma = live[dy] ? mask_a : 0u, mb = live[dy] ? mask_b : 0u;
          acc_a = __builtin_amdgcn_sad_u8(c4[dy] & ma, pred & ma, acc_a);
          acc_b = __builtin_amdgcn_sad_u8(c4[dy] & mb, pred & mb, acc_b);
        }
      }
    }
    if (acc_a) atomicAdd(&s_sum[col_a], acc_a);
    if (acc_b) atomicAdd(&s_sum[col_b], acc_b);
  }
  __syncthreads();
  uint32_t* out = p.res + (static_cast<int64_t>(frame) * p.grid_h + band) * p.grid_w;
  for (int i = tid; i < p.grid_w; i += 256)
    if (s_sum[i]) atomicAdd(out + i, s_sum[i]);
}

__global__ __launch_bounds__(256) void residual_mean_kernel(ResidualParams p) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int n_patch = p.grid_h * p.grid_w;
  if (i >= static_cast<int64_t>(p.n_frames) * n_patch) return;
  const int cell = static_cast<int>(i % n_patch);
  const int r = cell / p.grid_w, c = cell - r * p.grid_w;
  const int64_t wide = first_coord(c + 1, p.den_x, p.in_w, p.src_w) - first_coord(c, p.den_x, p.in_w, p.src_w);
  const int64_t tall = first_coord(r + 1, p.den_y, p.in_h, p.src_h) - first_coord(r, p.den_y, p.in_h, p.src_h);
  const unsigned long long n = static_cast<unsigned long long>(wide * tall);
  p.res[i] = n ? static_cast<uint32_t>((256ull * p.res[i]) / n) : 0u;
}

}  // namespace

extern "C" int cs_residual_proxy(const uint8_t* cur, const uint8_t* prev, const int16_t* mv_field,
                                 int32_t n_frames, int32_t src_w, int32_t src_h, int64_t pitch,
                                 int64_t frame_stride, int32_t cell, int32_t in_w, int32_t in_h,
                                 int32_t patch, int32_t grid_h, int32_t grid_w, uint32_t* res,
                                 void* stream) {
  if (n_frames < 0 || src_w < 1 || src_h < 1 || in_w < 1 || in_h < 1 || patch < 1 || grid_h < 1 || grid_w < 1)
    return CS_EINVAL;
  if (pitch < src_w || frame_stride < pitch * src_h) return CS_EINVAL;
  if (n_frames == 0) return CS_OK;
  if (!cur || !prev || !mv_field || !res) return CS_EINVAL;
  if (cell != 4 && cell != 8 && cell != 16) return CS_EUNSUPPORTED;
  if (src_w > 16384 || src_h > 16384 || in_w > 16384 || in_h > 16384 || patch > 1024) return CS_EUNSUPPORTED;
  if (grid_w > 8192 || static_cast<int64_t>(n_frames) * grid_h * grid_w >= (1ll << 31)) return CS_EUNSUPPORTED;
  if (pitch % 16 || frame_stride % 16 || pitch < ((src_w + 15) / 16) * 16) return CS_EUNSUPPORTED;
  if (!cs::aligned16(cur) || !cs::aligned16(prev) || (reinterpret_cast<uintptr_t>(mv_field) & 3u) ||
      (reinterpret_cast<uintptr_t>(res) & 3u))
    return CS_EUNSUPPORTED;
  // a 4-pixel group may touch two patch columns at most: columns at least 4 source pixels wide
  if (static_cast<int64_t>(patch) * src_w < 4ll * in_w) return CS_EUNSUPPORTED;

  ResidualParams p;
  p.cur = cur;
  p.prev = prev;
  p.field = reinterpret_cast<const uint32_t*>(mv_field);
  p.res = res;
  p.pitch = pitch;
  p.frame_stride = frame_stride;
  p.n_frames = n_frames;
  p.src_w = src_w;
  p.src_h = src_h;
  p.cell_shift = cell == 4 ? 2 : cell == 8 ? 3 : 4;
  p.cells_w = (src_w + cell - 1) / cell;
  p.cells_h = (src_h + cell - 1) / cell;
  p.in_w = in_w;
  p.in_h = in_h;
  p.den_x = static_cast<uint32_t>(patch) * src_w;
  p.den_y = static_cast<uint32_t>(patch) * src_h;
  p.div_x = exact_div(p.den_x);
  p.grid_h = grid_h;
  p.grid_w = grid_w;
  // enough workgroups to fill the chip: split a patch row's source rows among n_sub workgroups
  const int64_t bands = static_cast<int64_t>(n_frames) * grid_h;
  const int64_t band_rows = (static_cast<int64_t>(p.den_y) + in_h - 1) / in_h + 1;
  int64_t n_sub = (8192 + bands - 1) / bands;               // a few rounds of workgroups per CU
  if (n_sub > band_rows / 16) n_sub = band_rows / 16;        // at least four quads of rows each: the per-thread set-up is paid once per workgroup
  if (n_sub < 1) n_sub = 1;
  p.n_sub = static_cast<int32_t>(n_sub);
  if (bands * n_sub >= (1ll << 31)) return CS_EUNSUPPORTED;

  hipStream_t st = cs::as_stream(stream);
  const int64_t n_out = static_cast<int64_t>(n_frames) * grid_h * grid_w;
  hipLaunchKernelGGL(clear_sums_kernel, dim3(static_cast<unsigned>((n_out + 255) / 256)), dim3(256), 0, st, res, n_out);
  hipLaunchKernelGGL(residual_sum_kernel, dim3(static_cast<unsigned>(bands * n_sub)), dim3(256),
                     static_cast<size_t>(grid_w) * sizeof(uint32_t), st, p);
  hipLaunchKernelGGL(residual_mean_kernel, dim3(static_cast<unsigned>((n_out + 255) / 256)), dim3(256), 0, st, p);
  return cs::note_hip(hipGetLastError());
}
