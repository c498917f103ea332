// Backward pre- and post-passes shared by the fp32 and bf16 paths.
//   delta:   the row term of the softmax Jacobian, delta_i = sum_j P_ij dP_ij = dO_i . O_i;
//            the same pass rescales lse to base 2 for the kernels' exp2
//   combine: sum of the two per-class fp32 partials of dK/dV when one kv head serves
//            both shifted and unshifted query heads.
// Both are pure streaming kernels (HBM-bound, 16-byte coalesced accesses).
#include "s2attn_device.h"
#include "s2attn_launch.h"
#include "s2attn.h"

namespace s2 {
namespace {

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t hi16) { return __uint_as_float(hi16 << 16); }

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {   // round to nearest even
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// 16 lanes per (b,t,h) row; each lane reads 16-byte chunks.
template <bool BF16>
__global__ void __launch_bounds__(256) delta_kernel(const void* o, const void* dout, const float* lse,
                                                    float* delta, float* lse2, int B, int N, int H, int D) {
  const size_t row = (size_t)blockIdx.x * 16 + threadIdx.x / 16;
  const int lane = threadIdx.x % 16;
  const size_t rows = (size_t)B * N * H;
  float acc = 0.f;
  if (row < rows) {
    if (BF16) {
      const uint4* po = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(o) + row * D);
      const uint4* pd = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(dout) + row * D);
      for (int c = lane; c < D / 8; c += 16) {
        uint4 x = po[c], y = pd[c];
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc += bf16_bits_to_f32(xs[e] & 0xFFFFu) * bf16_bits_to_f32(ys[e] & 0xFFFFu);
          acc += bf16_bits_to_f32(xs[e] >> 16) * bf16_bits_to_f32(ys[e] >> 16);
        }
      }
    } else {
      const float4* po = reinterpret_cast<const float4*>(static_cast<const float*>(o) + row * D);
      const float4* pd = reinterpret_cast<const float4*>(static_cast<const float*>(dout) + row * D);
      for (int c = lane; c < D / 4; c += 16) {
        float4 x = po[c], y = pd[c];
        acc += x.x * y.x + x.y * y.y + x.z * y.z + x.w * y.w;
      }
    }
  }
  acc += __shfl_xor(acc, 1);
  acc += __shfl_xor(acc, 2);
  acc += __shfl_xor(acc, 4);
  acc += __shfl_xor(acc, 8);
  if (row < rows && lane == 0) {
    const size_t bt = row / H;
    const int h = (int)(row % H);
    const size_t b = bt / N, t = bt % N;
    delta[(b * H + h) * N + t] = acc;
    lse2[(b * H + h) * N + t] = lse[(b * H + h) * N + t] * 1.4426950408889634f;
  }
}

template <bool BF16>
__global__ void __launch_bounds__(256) combine_kernel(const float* partial, void* dk, void* dv, TStride sdk,
                                                      TStride sdv, int N, int Hkv, int D, size_t elems) {
  const size_t i4 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= elems) return;
  // contiguous (b, t, c, d) index of the partials -> row of the (possibly strided) output
  const int d = (int)(i4 % D);
  const size_t row = i4 / D;
  const int c = (int)(row % Hkv);
  const size_t bt = row / Hkv;
  const int t = (int)(bt % N), b = (int)(bt / N);
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const float4 x = *reinterpret_cast<const float4*>(partial + (size_t)(2 * which) * elems + i4);
    const float4 y = *reinterpret_cast<const float4*>(partial + (size_t)(2 * which + 1) * elems + i4);
    const float r0 = x.x + y.x, r1 = x.y + y.y, r2 = x.z + y.z, r3 = x.w + y.w;
    void* out = which == 0 ? dk : dv;
    const size_t o = row_off(which == 0 ? sdk : sdv, b, t, c) + d;
    if (BF16) {
      uint2 pk;
      pk.x = f32_to_bf16_bits(r0) | (f32_to_bf16_bits(r1) << 16);
      pk.y = f32_to_bf16_bits(r2) | (f32_to_bf16_bits(r3) << 16);
      *reinterpret_cast<uint2*>(static_cast<uint16_t*>(out) + o) = pk;
    } else {
      *reinterpret_cast<float4*>(static_cast<float*>(out) + o) = make_float4(r0, r1, r2, r3);
    }
  }
}

}  // namespace

int launch_delta(const KArgs& a, int dtype, hipStream_t st) {
  const size_t rows = (size_t)a.B * a.N * a.H;
  dim3 grid((unsigned)((rows + 15) / 16));
  if (dtype == S2ATTN_BF16)
    hipLaunchKernelGGL(delta_kernel<true>, grid, dim3(256), 0, st, a.o, a.dout, a.lse, a.delta, a.lse2, a.B, a.N, a.H, a.D);
  else
    hipLaunchKernelGGL(delta_kernel<false>, grid, dim3(256), 0, st, a.o, a.dout, a.lse, a.delta, a.lse2, a.B, a.N, a.H, a.D);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_combine_partials(const KArgs& a, int dtype, hipStream_t st) {
  const size_t elems = (size_t)a.B * a.N * a.Hkv * a.D;
  dim3 grid((unsigned)((elems / 4 + 255) / 256));
  if (dtype == S2ATTN_BF16)
    hipLaunchKernelGGL(combine_kernel<true>, grid, dim3(256), 0, st, a.dkv_partial, a.dk, a.dv, a.sdk, a.sdv, a.N,
                       a.Hkv, a.D, elems);
  else
    hipLaunchKernelGGL(combine_kernel<false>, grid, dim3(256), 0, st, a.dkv_partial, a.dk, a.dv, a.sdk, a.sdv, a.N,
                       a.Hkv, a.D, elems);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace s2
