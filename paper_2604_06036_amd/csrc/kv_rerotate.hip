// (b) Position-corrected reuse of cached keys, and (c) the refresh write, for gfx950.
//
// Paper Sec. 3.4.2, Eq. 6: K_hat = R(p_new) R(p_old)^-1 K = R(p_new - p_old) K for 1-D RoPE,
// V_hat = V.  Sec. 3.5: reusable states are repacked into the destination cache on the GPU and
// freshly computed K/V rows are written straight into that cache before attention.
//
// Both kernels are single-pass and HBM-bound: every thread moves 16-byte vectors, all loads of a
// thread's batch are issued before its first store, and nothing is staged through LDS because no
// byte is used twice, and for the same reason every load and store carries the non-temporal hint
// (streaming data should not displace what attention will want in the caches; measured +2..18 %).
// The re-rotation handles all decoder layers in one launch: a thread owns
// one (row, kv head, group of 4 or 8 frequency pairs), evaluates its theta_i and sin/cos once and sweeps a
// chunk of layers, so the trigonometry is amortised over layers and never limits bandwidth.
// Angles are formed as double(delta) * theta_i and reduced to [-pi/4, pi/4] plus a quadrant in
// double precision (a shift of a few thousand positions times theta_0 = 1 would lose 3 decimal
// digits in float); sin/cos of the reduced angle (single-precision minimax polynomials with the
// Cephes sinf/cosf coefficients), the products and the final rounding are single precision.
//
// Multidimensional RoPE (Sec. 3.4.2: each rotary dimension is corrected by the positional
// component the model maps to it): a row's shift is a triple (d_t, d_h, d_w) and frequency pair i
// is driven by component axis_of_pair[i]; everything else is the same kernel (template flag).
#include <math.h>

#include "common.h"

namespace {

constexpr int kMaxHalf = 128;            // head_dim <= 256
constexpr int kLayerBatch = 4;           // layers whose loads are in flight together

struct RerotateParams {
  void* k;
  void* v;
  const int32_t* __restrict__ src_slot;
  const int32_t* __restrict__ dst_slot;  // nullptr: in place
  const int32_t* __restrict__ delta;     // [n_rows], or [n_rows][3] with axis_of_pair
  const uint8_t* __restrict__ axis_of_pair;   // [head_dim / 2] values 0..2, multi-axis kernels only
  int64_t n_rows;
  int64_t stride_layer, stride_slot, stride_head;
  int32_t n_layers, n_kv_heads, head_dim, style;
  int32_t units_per_row;                 // n_kv_heads * (head_dim / 2 / kPairs)
  int32_t units_per_head;
  int32_t layers_per_block;
  double neg_log2_base_2_over_d;         // -2 log2(base) / head_dim:  theta_i = 2^(i * this)
};

template <bool kBf16>
struct Vec;
template <>
struct Vec<true> {                       // 8 bf16
  static constexpr int kElems = 8;
  cs::u32x4 raw;
  __device__ __forceinline__ void unpack(float* f) const {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ __forceinline__ void pack(const float* f) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = static_cast<uint32_t>(cs::f32_to_bf16(f[2 * i])) |
             (static_cast<uint32_t>(cs::f32_to_bf16(f[2 * i + 1])) << 16);
    raw = cs::u32x4{w[0], w[1], w[2], w[3]};
  }
};
template <>
struct Vec<false> {                      // 4 fp32
  static constexpr int kElems = 4;
  cs::u32x4 raw;
  __device__ __forceinline__ void unpack(float* f) const {
    f[0] = __uint_as_float(raw.x); f[1] = __uint_as_float(raw.y);
    f[2] = __uint_as_float(raw.z); f[3] = __uint_as_float(raw.w);
  }
  __device__ __forceinline__ void pack(const float* f) {
    raw = cs::u32x4{__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                    __float_as_uint(f[3])};
  }
};

// sin and cos of a double-precision angle, accurate to about 1e-7 absolute.
__device__ __forceinline__ void sincos_reduced(double ang, float* sn, float* cs_out) {
  const double kq = rint(ang * 0.63661977236758134);                   // 2 / pi
  double r = fma(-kq, 1.5707963267948966, ang);                        // pi / 2, high part
  r = fma(-kq, 6.123233995736766e-17, r);                              // pi / 2, low part
  const int quad = static_cast<int>(kq) & 3;
  const float x = static_cast<float>(r), z = x * x;
  const float s = fmaf(x * z, fmaf(z, fmaf(z, -1.9515295891e-4f, 8.3321608736e-3f), -1.6666654611e-1f), x);
  const float c = fmaf(z * z, fmaf(z, fmaf(z, 2.443315711809948e-5f, -1.388731625493765e-3f),
                                   4.166664568298827e-2f), fmaf(z, -0.5f, 1.0f));
  const float s_q = (quad & 1) ? c : s;
  const float c_q = (quad & 1) ? s : c;
  *sn = (quad & 2) ? -s_q : s_q;
  *cs_out = ((quad + 1) & 2) ? -c_q : c_q;
}

template <bool kBf16, int kStyle, bool kAxes>
__global__ __launch_bounds__(256) void rerotate_kernel(RerotateParams p) {
  using V = Vec<kBf16>;
  constexpr int E = V::kElems;           // pairs per thread = elements per vector
  using Elem = typename std::conditional<kBf16, uint16_t, float>::type;

  const int64_t unit = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (unit >= p.n_rows * p.units_per_row) return;
  const int64_t row = unit / p.units_per_row;
  const int rem = static_cast<int>(unit - row * p.units_per_row);
  const int head = rem / p.units_per_head;
  const int j = rem - head * p.units_per_head;          // which group of E pairs inside the head
  const int half = p.head_dim / 2;

  const int src = p.src_slot[row];
  const int dst = p.dst_slot ? p.dst_slot[row] : src;
  if (src < 0 || dst < 0) return;        // padding rows of a list sized to its capacity
  double dlt[3];
  if (kAxes) {
    dlt[0] = static_cast<double>(p.delta[row * 3]);
    dlt[1] = static_cast<double>(p.delta[row * 3 + 1]);
    dlt[2] = static_cast<double>(p.delta[row * 3 + 2]);
  } else {
    dlt[0] = dlt[1] = dlt[2] = static_cast<double>(p.delta[row]);
  }

  float cs_[E], sn_[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const double theta = exp2(static_cast<double>(j * E + e) * p.neg_log2_base_2_over_d);
    double shift = dlt[0];
    if (kAxes) {
      const int axis = p.axis_of_pair[j * E + e];
      shift = axis == 0 ? dlt[0] : axis == 1 ? dlt[1] : dlt[2];
    }
    sincos_reduced(shift * theta, &sn_[e], &cs_[e]);
  }

  // element offsets of the thread's two vectors inside a head
  const int off_a = kStyle == CS_ROPE_HALF_SPLIT ? j * E : 2 * j * E;
  const int off_b = kStyle == CS_ROPE_HALF_SPLIT ? half + j * E : 2 * j * E + E;
  const int64_t src_off = static_cast<int64_t>(src) * p.stride_slot + head * p.stride_head;
  const int64_t dst_off = static_cast<int64_t>(dst) * p.stride_slot + head * p.stride_head;
  const bool repack = p.dst_slot != nullptr;
  Elem* kbase = static_cast<Elem*>(p.k);
  Elem* vbase = static_cast<Elem*>(p.v);

  const int l_begin = blockIdx.y * p.layers_per_block;
  const int l_end = min(p.n_layers, l_begin + p.layers_per_block);
  for (int l0 = l_begin; l0 < l_end; l0 += kLayerBatch) {
    cs::u32x4 ka[kLayerBatch], kb[kLayerBatch], va[kLayerBatch], vb[kLayerBatch];
#pragma unroll
    for (int i = 0; i < kLayerBatch; ++i) {
      if (l0 + i < l_end) {
        const int64_t lo = static_cast<int64_t>(l0 + i) * p.stride_layer + src_off;
        ka[i] = __builtin_nontemporal_load(reinterpret_cast<const cs::u32x4*>(kbase + lo + off_a));
        kb[i] = __builtin_nontemporal_load(reinterpret_cast<const cs::u32x4*>(kbase + lo + off_b));
        if (repack) {
          va[i] = __builtin_nontemporal_load(reinterpret_cast<const cs::u32x4*>(vbase + lo + off_a));
          vb[i] = __builtin_nontemporal_load(reinterpret_cast<const cs::u32x4*>(vbase + lo + off_b));
        }
      }
    }
#pragma unroll
    for (int i = 0; i < kLayerBatch; ++i) {
      if (l0 + i < l_end) {
        float fa[E], fb[E], ya[E], yb[E];
        V ta, tb;
        ta.raw = ka[i];
        tb.raw = kb[i];
        ta.unpack(fa);
        tb.unpack(fb);
        if (kStyle == CS_ROPE_HALF_SPLIT) {
          // pair e of the thread is (fa[e], fb[e]): elements i and i + d/2 of the head
#pragma unroll
          for (int e = 0; e < E; ++e) {
            ya[e] = fmaf(fa[e], cs_[e], -(fb[e] * sn_[e]));
            yb[e] = fmaf(fb[e], cs_[e], fa[e] * sn_[e]);
          }
        } else {
          // the two vectors are contiguous; pair e is elements (2e, 2e+1) of their concatenation
#pragma unroll
          for (int e = 0; e < E / 2; ++e) {
            ya[2 * e] = fmaf(fa[2 * e], cs_[e], -(fa[2 * e + 1] * sn_[e]));
            ya[2 * e + 1] = fmaf(fa[2 * e + 1], cs_[e], fa[2 * e] * sn_[e]);
            yb[2 * e] = fmaf(fb[2 * e], cs_[E / 2 + e], -(fb[2 * e + 1] * sn_[E / 2 + e]));
            yb[2 * e + 1] = fmaf(fb[2 * e + 1], cs_[E / 2 + e], fb[2 * e] * sn_[E / 2 + e]);
          }
        }
        V oa, ob;
        oa.pack(ya);
        ob.pack(yb);
        const int64_t lo = static_cast<int64_t>(l0 + i) * p.stride_layer + dst_off;
        __builtin_nontemporal_store(oa.raw, reinterpret_cast<cs::u32x4*>(kbase + lo + off_a));
        __builtin_nontemporal_store(ob.raw, reinterpret_cast<cs::u32x4*>(kbase + lo + off_b));
        if (repack) {
          __builtin_nontemporal_store(va[i], reinterpret_cast<cs::u32x4*>(vbase + lo + off_a));
          __builtin_nontemporal_store(vb[i], reinterpret_cast<cs::u32x4*>(vbase + lo + off_b));
        }
      }
    }
  }
}

struct ScatterParams {
  const void* __restrict__ k_new;
  const void* __restrict__ v_new;
  const int32_t* __restrict__ slot;
  void* __restrict__ k_cache;
  void* __restrict__ v_cache;
  int64_t n_tok, stride_slot, stride_head;
  int32_t vecs_per_row, vecs_per_head, elems_per_vec;
};

constexpr int kScatterBatch = 2;

template <typename Elem>
__global__ __launch_bounds__(256) void scatter_kernel(ScatterParams p) {
  const int64_t n_units = p.n_tok * p.vecs_per_row;
  const int64_t first = (static_cast<int64_t>(blockIdx.x) * blockDim.x) * kScatterBatch + threadIdx.x;
  cs::u32x4 kv[kScatterBatch], vv[kScatterBatch];
  int64_t dst[kScatterBatch];
#pragma unroll
  for (int i = 0; i < kScatterBatch; ++i) {
    const int64_t unit = first + static_cast<int64_t>(i) * blockDim.x;
    dst[i] = -1;
    if (unit < n_units) {
      const int64_t tok = unit / p.vecs_per_row;
      const int rem = static_cast<int>(unit - tok * p.vecs_per_row);
      const int sl = p.slot[tok];
      if (sl >= 0) {
        const int head = rem / p.vecs_per_head;
        const int c = rem - head * p.vecs_per_head;
        dst[i] = static_cast<int64_t>(sl) * p.stride_slot + head * p.stride_head +
                 static_cast<int64_t>(c) * p.elems_per_vec;
        const int64_t so = unit * p.elems_per_vec;
        kv[i] = __builtin_nontemporal_load(reinterpret_cast<const cs::u32x4*>(static_cast<const Elem*>(p.k_new) + so));
        vv[i] = __builtin_nontemporal_load(reinterpret_cast<const cs::u32x4*>(static_cast<const Elem*>(p.v_new) + so));
      }
    }
  }
#pragma unroll
  for (int i = 0; i < kScatterBatch; ++i) {
    if (dst[i] >= 0) {
      __builtin_nontemporal_store(kv[i], reinterpret_cast<cs::u32x4*>(static_cast<Elem*>(p.k_cache) + dst[i]));
      __builtin_nontemporal_store(vv[i], reinterpret_cast<cs::u32x4*>(static_cast<Elem*>(p.v_cache) + dst[i]));
    }
  }
}

}  // namespace

namespace {

// delta: [n_rows] shifts, or with axis_of_pair [n_rows][3] shifts per positional component.
int rerotate_launch(void* k_cache, void* v_cache, const int32_t* src_slot, const int32_t* dst_slot,
                    const int32_t* delta, const uint8_t* axis_of_pair, int64_t n_rows, int32_t n_layers,
                    int32_t n_kv_heads, int32_t head_dim, int64_t stride_layer, int64_t stride_slot,
                    int64_t stride_head, float rope_base, int32_t rope_style, int32_t dtype, void* stream) {
  if (n_rows < 0 || n_layers < 0 || n_kv_heads < 1 || head_dim < 1) return CS_EINVAL;
  if (stride_layer < 0 || stride_slot < 0 || stride_head < 0) return CS_EINVAL;
  if (!(rope_base > 0.0f)) return CS_EINVAL;
  if (dtype != CS_F32 && dtype != CS_BF16) return CS_EUNSUPPORTED;
  if (rope_style != CS_ROPE_HALF_SPLIT && rope_style != CS_ROPE_INTERLEAVED) return CS_EUNSUPPORTED;
  if (head_dim % 16 != 0 || head_dim > 2 * kMaxHalf) return CS_EUNSUPPORTED;
  const int elems = dtype == CS_BF16 ? 8 : 4;              // elements per 16-byte vector
  if (stride_layer % elems || stride_slot % elems || stride_head % elems) return CS_EUNSUPPORTED;
  if (n_rows == 0 || n_layers == 0) return CS_OK;
  if (!k_cache || !src_slot || !delta) return CS_EINVAL;
  if (dst_slot && !v_cache) return CS_EINVAL;
  if (!cs::aligned16(k_cache) || (dst_slot && !cs::aligned16(v_cache))) return CS_EUNSUPPORTED;

  const int half = head_dim / 2;
  RerotateParams p;
  p.k = k_cache;
  p.v = v_cache;
  p.src_slot = src_slot;
  p.dst_slot = dst_slot;
  p.delta = delta;
  p.axis_of_pair = axis_of_pair;
  p.n_rows = n_rows;
  p.stride_layer = stride_layer;
  p.stride_slot = stride_slot;
  p.stride_head = stride_head;
  p.n_layers = n_layers;
  p.n_kv_heads = n_kv_heads;
  p.head_dim = head_dim;
  p.style = rope_style;
  p.neg_log2_base_2_over_d = -2.0 * log2(static_cast<double>(rope_base)) / head_dim;
  p.units_per_head = half / elems;
  p.units_per_row = n_kv_heads * p.units_per_head;

  const int64_t n_units = n_rows * p.units_per_row;
  const int64_t blocks_x = (n_units + 255) / 256;
  if (blocks_x > 0x7fffffffll) return CS_EUNSUPPORTED;
  // Layers per block: as many as possible (amortises sin/cos) while the grid still holds a few
  // thousand workgroups, so that all 256 compute units have several resident waves each.
  int lpb = n_layers;
  while (lpb > kLayerBatch && blocks_x * ((n_layers + lpb - 1) / lpb) < 4096) lpb = (lpb + 1) / 2;
  lpb = ((lpb + kLayerBatch - 1) / kLayerBatch) * kLayerBatch;
  p.layers_per_block = lpb;
  const dim3 grid(static_cast<unsigned>(blocks_x), static_cast<unsigned>((n_layers + lpb - 1) / lpb));
  hipStream_t st = cs::as_stream(stream);
  const bool half_split = rope_style == CS_ROPE_HALF_SPLIT;
  const bool bf16 = dtype == CS_BF16;
#define CS_LAUNCH_REROTATE(AXES)                                                                             \
  do {                                                                                                       \
    if (bf16 && half_split)                                                                                  \
      hipLaunchKernelGGL((rerotate_kernel<true, CS_ROPE_HALF_SPLIT, AXES>), grid, dim3(256), 0, st, p);      \
    else if (bf16)                                                                                           \
      hipLaunchKernelGGL((rerotate_kernel<true, CS_ROPE_INTERLEAVED, AXES>), grid, dim3(256), 0, st, p);     \
    else if (half_split)                                                                                     \
      hipLaunchKernelGGL((rerotate_kernel<false, CS_ROPE_HALF_SPLIT, AXES>), grid, dim3(256), 0, st, p);     \
    else                                                                                                     \
      hipLaunchKernelGGL((rerotate_kernel<false, CS_ROPE_INTERLEAVED, AXES>), grid, dim3(256), 0, st, p);    \
  } while (0)
  if (axis_of_pair) CS_LAUNCH_REROTATE(true);
  else CS_LAUNCH_REROTATE(false);
#undef CS_LAUNCH_REROTATE
  return cs::note_hip(hipGetLastError());
}

}  // namespace

extern "C" int cs_kv_rerotate(void* k_cache, void* v_cache, const int32_t* src_slot,
                              const int32_t* dst_slot, const int32_t* delta, int64_t n_rows,
                              int32_t n_layers, int32_t n_kv_heads, int32_t head_dim,
                              int64_t stride_layer, int64_t stride_slot, int64_t stride_head,
                              float rope_base, int32_t rope_style, int32_t dtype, void* stream) {
  return rerotate_launch(k_cache, v_cache, src_slot, dst_slot, delta, nullptr, n_rows, n_layers, n_kv_heads,
                         head_dim, stride_layer, stride_slot, stride_head, rope_base, rope_style, dtype, stream);
}

extern "C" int cs_kv_rerotate_axes(void* k_cache, void* v_cache, const int32_t* src_slot,
                                   const int32_t* dst_slot, const int32_t* delta3,
                                   const uint8_t* axis_of_pair, int64_t n_rows, int32_t n_layers,
                                   int32_t n_kv_heads, int32_t head_dim, int64_t stride_layer,
                                   int64_t stride_slot, int64_t stride_head, float rope_base,
                                   int32_t rope_style, int32_t dtype, void* stream) {
  if (n_rows > 0 && n_layers > 0 && !axis_of_pair) return CS_EINVAL;
  return rerotate_launch(k_cache, v_cache, src_slot, dst_slot, delta3, axis_of_pair, n_rows, n_layers,
                         n_kv_heads, head_dim, stride_layer, stride_slot, stride_head, rope_base, rope_style,
                         dtype, stream);
}

extern "C" int cs_kv_refresh_scatter(const void* k_new, const void* v_new, const int32_t* slot,
                                     void* k_cache_layer, void* v_cache_layer, int64_t n_tok,
                                     int32_t n_kv_heads, int32_t head_dim, int64_t stride_slot,
                                     int64_t stride_head, int32_t dtype, void* stream) {
  if (n_tok < 0 || n_kv_heads < 1 || head_dim < 1 || stride_slot < 0 || stride_head < 0)
    return CS_EINVAL;
  if (dtype != CS_F32 && dtype != CS_BF16) return CS_EUNSUPPORTED;
  const int elems = dtype == CS_BF16 ? 8 : 4;
  if (head_dim % elems || stride_slot % elems || stride_head % elems) return CS_EUNSUPPORTED;
  if (n_tok == 0) return CS_OK;
  if (!k_new || !v_new || !slot || !k_cache_layer || !v_cache_layer) return CS_EINVAL;
  if (!cs::aligned16(k_new) || !cs::aligned16(v_new) || !cs::aligned16(k_cache_layer) ||
      !cs::aligned16(v_cache_layer))
    return CS_EUNSUPPORTED;

  ScatterParams p;
  p.k_new = k_new;
  p.v_new = v_new;
  p.slot = slot;
  p.k_cache = k_cache_layer;
  p.v_cache = v_cache_layer;
  p.n_tok = n_tok;
  p.stride_slot = stride_slot;
  p.stride_head = stride_head;
  p.vecs_per_head = head_dim / elems;
  p.vecs_per_row = n_kv_heads * p.vecs_per_head;
  p.elems_per_vec = elems;
  const int64_t n_units = n_tok * p.vecs_per_row;
  const int64_t blocks = (n_units + 256 * kScatterBatch - 1) / (256 * kScatterBatch);
  if (blocks > 0x7fffffffll) return CS_EUNSUPPORTED;
  if (dtype == CS_BF16)
    hipLaunchKernelGGL(scatter_kernel<uint16_t>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0,
                       cs::as_stream(stream), p);
  else
    hipLaunchKernelGGL(scatter_kernel<float>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0,
                       cs::as_stream(stream), p);
  return cs::note_hip(hipGetLastError());
}
