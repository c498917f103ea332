// Hardware probes behind the design notes of the S2-Attn kernels (gfx950).  Not part of the
// attention path: a separate small library (libs2attn_probes.so) that bench.py --probes
// runs, so that the figures the kernel design leans on can be re-measured on any box:
//   * the bf16 32x32x16 MFMA rate a compute unit sustains as a function of the operand
//     DATA (the chip is power-limited: random operands run slower than constant ones),
//     with operands in registers, and with one operand fragment per MFMA read from LDS in
//     the kernels' swizzled tile layout, with and without softmax-like vector work;
//   * the rate at which the L2 performs fp32 atomic adds in the access pattern a fused
//     backward would use to accumulate dQ partial tiles.
// Every probe allocates its own small buffers, times its launches with HIP events on the
// default stream and returns 0 or the failing hipError_t.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstring>
#include <random>
#include <type_traits>
#include <vector>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define S2P_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))
#define S2P_CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return (int)e_; } while (0)

__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
__device__ __forceinline__ int tile_off(int row, int chunk) { return row * 256 + ((chunk ^ swz(row)) << 4); }

uint16_t to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  u += 0x7fff + ((u >> 16) & 1);
  return (uint16_t)(u >> 16);
}

// data_mode: 0 = all ones, 1 = iid N(0,1)
std::vector<uint16_t> operand_data(size_t n, int data_mode) {
  std::vector<uint16_t> h(n);
  std::mt19937 rng(1);
  std::normal_distribution<float> nd(0.f, 1.f);
  for (auto& x : h) x = to_bf16(data_mode == 0 ? 1.0f : nd(rng));
  return h;
}

// ---- MFMAs on register operands only: every MFMA takes a new A and a new B fragment.
__global__ void __launch_bounds__(256) mfma_registers_kernel(const bf16x8* __restrict__ src, float* out, int iters) {
  __shared__ char pad[98304];   // more than half of the CU's LDS: one workgroup (one wave per SIMD) per CU
  if (iters < 0) pad[threadIdx.x] = 1;
  const int lane = threadIdx.x & 63;
  bf16x8 A[8], B[8];
  for (int j = 0; j < 8; ++j) { A[j] = src[j * 64 + lane]; B[j] = src[(8 + j) * 64 + lane]; }
  f32x16 c[4];
  for (int i = 0; i < 4; i++) for (int v = 0; v < 16; v++) c[i][v] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      c[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[j], B[j], c[0], 0, 0, 0);
      c[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[(j + 1) & 7], B[(j + 3) & 7], c[1], 0, 0, 0);
      c[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[(j + 2) & 7], B[(j + 5) & 7], c[2], 0, 0, 0);
      c[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[(j + 3) & 7], B[(j + 7) & 7], c[3], 0, 0, 0);
    }
  }
  float s = 0;
  for (int i = 0; i < 4; i++) for (int v = 0; v < 16; v++) s += c[i][v];
  out[blockIdx.x * 256 + threadIdx.x] = s + (iters < 0 ? pad[lane] : 0);
}

// ---- Every MFMA takes its A operand from LDS (one 1 KB fragment per MFMA, in the tile layout
// of the attention kernels), B from registers.  TR: row-major ds_read_b128 fragments (0) or
// transposing 2 x ds_read_b64_tr_b16 (1).  KV fused multiply-adds and EV exp2 per MFMA stand for
// the softmax work.  Fragments are fetched two steps (8 MFMAs) ahead.  REUSE = 2: only two
// fragments are read per step and each feeds two MFMAs (against two register operands), the
// LDS traffic of a kernel whose waves own twice as many rows.
template <int TR, int KV, int EV, int REUSE = 1>
__global__ void __launch_bounds__(512) mfma_lds_kernel(float* out, int iters, const uint32_t* __restrict__ src) {
  __shared__ __attribute__((aligned(1024))) char lds[65536 + 32768];   // one workgroup per CU
  for (int i = threadIdx.x; i < 16384; i += blockDim.x) ((uint32_t*)lds)[i] = src[i];
  __syncthreads();
  const int lane = threadIdx.x & 63, l32 = lane & 31, g32 = lane >> 5;
  int orm[8], otr[8];
  for (int k = 0; k < 8; ++k) orm[k] = tile_off(l32, 2 * k + g32);
  {
    const int L = lane & 15, half = lane & 16;
    const int row = 4 * g32 + (L >> 2);
    for (int cb = 0; cb < 4; ++cb) {
      const int col = 32 * cb + half + 4 * (L & 3);
      const int chunk = col >> 3, within = (col & 7) * 2;
      otr[2 * cb] = row * 256 + ((chunk ^ swz(row)) << 4) + within;
      otr[2 * cb + 1] = (row + 8) * 256 + ((chunk ^ swz(row + 8)) << 4) + within;
    }
  }
  bf16x8 b = *reinterpret_cast<const bf16x8*>(src + 4 * (threadIdx.x & 63));
  bf16x8 b2 = *reinterpret_cast<const bf16x8*>(src + 4 * (64 + (threadIdx.x & 63)));
  f32x16 c[4];
  for (int i = 0; i < 4; i++) for (int v = 0; v < 16; v++) c[i][v] = 0;
  auto load = [&](bf16x8 (&buf)[4], auto stepc, int tsel) {
    constexpr int ST = decltype(stepc)::value;   // 0..3 within a tile
    const char* tile = lds + (tsel & 3) * 16384;
    if (TR == 0) {
#pragma unroll
      for (int i = 0; i < 4 / REUSE; ++i)
        buf[i] = *reinterpret_cast<const bf16x8*>(tile + orm[2 * ST + (i >> 1)] + (i & 1) * 32 * 256);
    } else {
#pragma unroll
      for (int i = 0; i < 4 / REUSE; ++i) {
        bf16x4 lo_ = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(S2P_LDS(bf16x4, tile + otr[2 * i] + ST * 16 * 256));
        bf16x4 hi_ = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(S2P_LDS(bf16x4, tile + otr[2 * i + 1] + ST * 16 * 256));
        buf[i] = __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    }
  };
  float x[16];
  for (int i = 0; i < 16; i++) x[i] = threadIdx.x * 0.001f + i * 0.01f;
  auto mma = [&](const bf16x8 (&buf)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(buf[REUSE == 2 ? i >> 1 : i], (REUSE == 2 && (i & 1)) ? b2 : b, c[i], 0, 0, 0);
#pragma unroll
      for (int t = 0; t < KV; t++) x[(i * KV + t) & 15] = fmaf(x[(i * KV + t) & 15], 0.999f, 0.001f);
#pragma unroll
      for (int t = 0; t < EV; t++) x[(i * EV + t + 8) & 15] = __builtin_amdgcn_exp2f(x[(i * EV + t + 8) & 15] * 0.5f - 1.0f);
    }
  };
  using std::integral_constant;
  bf16x8 f0[4], f1[4], f2[4];
  load(f0, integral_constant<int, 0>{}, 0);
  load(f1, integral_constant<int, 1>{}, 0);
  // 12 steps of 4 MFMAs per outer iteration: ring of 3 fragment buffers, 4 steps per tile
  for (int it = 0; it < iters; it += 12) {
    const int t = it >> 2;
#define S2P_STEP(A, B, C, S, T) load(C, integral_constant<int, (S + 2) & 3>{}, T + ((S + 2) >> 2)); mma(A); __builtin_amdgcn_sched_barrier(0);
    S2P_STEP(f0, f1, f2, 0, t)     S2P_STEP(f1, f2, f0, 1, t)     S2P_STEP(f2, f0, f1, 2, t)     S2P_STEP(f0, f1, f2, 3, t)
    S2P_STEP(f1, f2, f0, 0, t + 1) S2P_STEP(f2, f0, f1, 1, t + 1) S2P_STEP(f0, f1, f2, 2, t + 1) S2P_STEP(f1, f2, f0, 3, t + 1)
    S2P_STEP(f2, f0, f1, 0, t + 2) S2P_STEP(f0, f1, f2, 1, t + 2) S2P_STEP(f1, f2, f0, 2, t + 2) S2P_STEP(f2, f0, f1, 3, t + 2)
#undef S2P_STEP
  }
  float s = 0;
  for (int i = 0; i < 4; i++) for (int v = 0; v < 16; v++) s += c[i][v];
  for (int i = 0; i < 16; i++) s += x[i];
  for (int i = 0; i < 4 / REUSE; ++i) for (int e = 0; e < 8; ++e) s += (float)f0[i][e] + (float)f1[i][e];
  out[blockIdx.x * 512 + threadIdx.x] = s;
}

// ---- fp32 atomic adds of 64-row x 128-float tiles (32 KB, what a workgroup of a fused
// backward would add into a dQ accumulation buffer for every (64 queries x 128 keys) tile):
// 256 workgroups, the 32 of an XCD walking the 128 tiles of one 4 MB region at a time.
__global__ void __launch_bounds__(512, 1) atomic_tiles_kernel(float* acc, int iters, int tiles_per_region, int regions) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int l32 = lane & 31, g = lane >> 5, qb = w >> 2;
  for (int it = 0; it < iters; ++it) {
    const int n = slot * 2 + it;   // tile sequence of a key tile: from its diagonal on, ascending
    const int region = xcd + 8 * ((n / tiles_per_region) % regions);
    float* base = acc + ((size_t)region * tiles_per_region + n % tiles_per_region) * (64 * 128);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = 32 * qb + 8 * (v / 4) + 4 * g + (v % 4);
      __hip_atomic_fetch_add(base + row * 128 + 32 * (w & 3) + l32, 1e-3f * (float)(v + 1 + lane), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

template <class Launch>
int time_launches(Launch launch, int reps, float* best_ms) {
  hipEvent_t e0, e1;
  S2P_CK(hipEventCreate(&e0));
  S2P_CK(hipEventCreate(&e1));
  *best_ms = 1e30f;
  for (int rep = 0; rep < reps; ++rep) {
    S2P_CK(hipEventRecord(e0, 0));
    launch();
    S2P_CK(hipGetLastError());
    S2P_CK(hipEventRecord(e1, 0));
    S2P_CK(hipEventSynchronize(e1));
    float ms = 0;
    S2P_CK(hipEventElapsedTime(&ms, e0, e1));
    if (rep > 0 && ms < *best_ms) *best_ms = ms;   // the first launch is the warm-up
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return 0;
}

}  // namespace

#define S2P_API extern "C" __attribute__((visibility("default")))

// Sustained TFLOP/s of a loop of nothing but MFMAs on register operands, one wave per SIMD on
// every CU.  data_mode: 0 = ones, 1 = N(0,1).
S2P_API int s2probe_mfma_registers(int data_mode, double* tflops) {
  const int n = 16 * 64 * 8, iters = 40000, nb = 256;
  const std::vector<uint16_t> h = operand_data(n, data_mode);
  bf16x8* d = nullptr;
  float* o = nullptr;
  S2P_CK(hipMalloc(&d, n * 2));
  S2P_CK(hipMalloc(&o, nb * 256 * 4));
  S2P_CK(hipMemcpy(d, h.data(), n * 2, hipMemcpyHostToDevice));
  float ms = 0;
  int rc = time_launches([&] { hipLaunchKernelGGL(mfma_registers_kernel, dim3(nb), dim3(256), 0, 0, d, o, iters); }, 4, &ms);
  (void)hipFree(d);
  (void)hipFree(o);
  if (rc) return rc;
  *tflops = (double)nb * 4 * iters * 32 * 32768.0 / ms / 1e9;
  return 0;
}

// Same with the A operand of every MFMA read from LDS.  transposed: 0 / 1; vector_work: 0 =
// none, 1 = 3 fma + 1 exp2 per MFMA, 2 = 4 fma + 2 exp2; waves_per_simd: 1 or 2; reuse: MFMAs
// fed by one LDS fragment, 1 or 2.
S2P_API int s2probe_mfma_lds(int transposed, int vector_work, int waves_per_simd, int reuse, int data_mode, double* tflops) {
  if (transposed < 0 || transposed > 1 || vector_work < 0 || vector_work > 2 || waves_per_simd < 1 || waves_per_simd > 2 ||
      reuse < 1 || reuse > 2)
    return (int)hipErrorInvalidValue;
  const int iters = 120000, nb = 256, threads = 256 * waves_per_simd;
  const std::vector<uint16_t> h = operand_data(32768, data_mode);
  uint32_t* src = nullptr;
  float* o = nullptr;
  S2P_CK(hipMalloc(&src, 65536));
  S2P_CK(hipMalloc(&o, nb * 512 * 4));
  S2P_CK(hipMemcpy(src, h.data(), 65536, hipMemcpyHostToDevice));
  float ms = 0;
  auto launch = [&] {
#define S2P_CASE(TR, VW, KV, EV) \
    if (transposed == TR && vector_work == VW && reuse == 1) hipLaunchKernelGGL((mfma_lds_kernel<TR, KV, EV, 1>), dim3(nb), dim3(threads), 0, 0, o, iters, src); \
    if (transposed == TR && vector_work == VW && reuse == 2) hipLaunchKernelGGL((mfma_lds_kernel<TR, KV, EV, 2>), dim3(nb), dim3(threads), 0, 0, o, iters, src);
    S2P_CASE(0, 0, 0, 0) S2P_CASE(0, 1, 3, 1) S2P_CASE(0, 2, 4, 2)
    S2P_CASE(1, 0, 0, 0) S2P_CASE(1, 1, 3, 1) S2P_CASE(1, 2, 4, 2)
#undef S2P_CASE
  };
  int rc = time_launches(launch, 3, &ms);
  (void)hipFree(src);
  (void)hipFree(o);
  if (rc) return rc;
  *tflops = (double)nb * (threads / 64) * iters * 4 * 32768.0 / ms / 1e9;
  return 0;
}

// TB/s of fp32 atomic adds (4 bytes counted per add) in the dQ-partial-tile pattern.
S2P_API int s2probe_atomic_add(double* tb_per_s) {
  const int tiles_per_region = 128, regions = 16, iters = 2048;
  const size_t n = (size_t)8 * regions * tiles_per_region * 64 * 128;   // 512 MB
  float* acc = nullptr;
  S2P_CK(hipMalloc(&acc, n * 4));
  S2P_CK(hipMemset(acc, 0, n * 4));
  float ms = 0;
  int rc = time_launches([&] { hipLaunchKernelGGL(atomic_tiles_kernel, dim3(256), dim3(512), 0, 0, acc, iters, tiles_per_region, regions); }, 3, &ms);
  (void)hipFree(acc);
  if (rc) return rc;
  *tb_per_s = 256.0 * iters * 32768.0 / ms / 1e9;
  return 0;
}
