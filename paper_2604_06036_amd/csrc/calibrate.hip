// Measurement aid, not part of the method: a kernel that issues nothing but bf16 matrix-core
// instructions (v_mfma_f32_32x32x16_bf16, four independent accumulators per wave, operands held in
// registers), so that bench.py can report what the matrix cores of THIS device sustain next to the
// published peak the attention kernel is priced against.  With lane-dependent pseudo-random operands
// the device settles at a lower clock (and inserts issue stalls) than with constant ones: the
// sustained rate of dense bf16 work on real data is the figure to read the attention fraction against.
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <bool kRandom>
__global__ __launch_bounds__(256, 2) void mfma_probe_kernel(float* sink, int32_t iters) {
  const uint32_t tid = threadIdx.x + blockIdx.x * 256u;
  uint32_t h1 = (tid * 2654435761u) ^ 0x9e3779b9u, h2 = (tid * 40503u + 77u) * 2246822519u;
  // bf16 pairs in +-[0.5, 1): xorshift bits under fixed exponents
  auto draw = [](uint32_t& x) {
    x ^= x << 13; x ^= x >> 17; x ^= x << 5;
    return kRandom ? ((x & 0x807f807fu) | 0x3f003f00u) : 0x3f803f80u;
  };
  bf16x8 a = __builtin_bit_cast(bf16x8, cs::u32x4{draw(h1), draw(h1), draw(h1), draw(h1)});
  bf16x8 b = __builtin_bit_cast(bf16x8, cs::u32x4{draw(h2), draw(h2), draw(h2), draw(h2)});
  f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int r = 0; r < 16; ++r) { c0[r] = 0.f; c1[r] = 0.f; c2[r] = 0.f; c3[r] = 0.f; }
  for (int it = 0; it < iters; ++it) {
    asm volatile("" : "+v"(a), "+v"(b));           // keeps the loop from being folded
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, a, c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, b, c3, 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
  if (s == 12345.678f) sink[tid] = s;               // never true: keeps the accumulators alive
}

}  // namespace

extern "C" int cs_mfma_rate_probe(float* sink, int32_t n_workgroups, int32_t iters, int32_t random_operands,
                                  void* stream) {
  if (!sink || n_workgroups < 1 || iters < 1 || n_workgroups > (1 << 20)) return CS_EINVAL;
  hipStream_t st = cs::as_stream(stream);
  if (random_operands)
    hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(n_workgroups), dim3(256), 0, st, sink, iters);
  else
    hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(n_workgroups), dim3(256), 0, st, sink, iters);
  return cs::note_hip(hipGetLastError());
}
