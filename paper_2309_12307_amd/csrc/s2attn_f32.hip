// fp32 S2-Attn kernels (forward, delta pre-pass, dK/dV, dQ) for gfx950.
//
// Plain LDS-tiled fp32 FMA kernels: every product and sum is fp32, so this mode
// serves the tight-tolerance configuration (LongLoRA Section 3.2 / Algorithm 1 at
// small shapes) and arbitrary even group sizes (partial tiles are masked).
// The shift and the grouping are pure row-address arithmetic (token_of); no rolled
// copy of q, k, v or o exists anywhere.
#include "s2attn_device.h"
#include "s2attn_launch.h"

namespace s2 {
namespace {

constexpr int kThreads = 256;
constexpr int BN = 64;   // keys per tile
constexpr int SLD = 65;  // leading dimension of score tiles in LDS

// Loads rows [i0, i0+ROWS) of group g (in-group order) of one head into LDS,
// zero-filling rows past the end of the group.
template <int ROWS, int D>
__device__ __forceinline__ void load_tile(float* dst, const float* src, const TStride& st, int b, int head,
                                          int g, int i0, int s, int N, int G) {
  constexpr int LD = D + 4;
  constexpr int C4 = D / 4;
  for (int idx = threadIdx.x; idx < ROWS * C4; idx += kThreads) {
    int row = idx / C4, c4 = idx % C4;
    int i = i0 + row;
    float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < G) {
      int tok = token_of(g * G + i, s, N);
      val = *reinterpret_cast<const float4*>(src + row_off(st, b, tok, head) + 4 * c4);
    }
    *reinterpret_cast<float4*>(dst + row * LD + 4 * c4) = val;
  }
}

// acc[a][b] = sum_d A[(ty+16a)][d] * Bm[(tx+16b)][d]   (A: RA*16 rows, Bm: 64 rows)
template <int RA, int D>
__device__ __forceinline__ void tile_nt(float (&acc)[RA][4], const float* A, const float* Bm, int ty, int tx) {
  constexpr int LD = D + 4;
#pragma unroll
  for (int a = 0; a < RA; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;
  for (int d = 0; d < D; d += 4) {
    float4 av[RA], bv[4];
#pragma unroll
    for (int a = 0; a < RA; ++a) av[a] = *reinterpret_cast<const float4*>(A + (ty + 16 * a) * LD + d);
#pragma unroll
    for (int b = 0; b < 4; ++b) bv[b] = *reinterpret_cast<const float4*>(Bm + (tx + 16 * b) * LD + d);
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b)
        acc[a][b] += av[a].x * bv[b].x + av[a].y * bv[b].y + av[a].z * bv[b].z + av[a].w * bv[b].w;
  }
}

// ---------------------------------------------------------------------------
// Forward: one block per (query tile of 64 rows, group, batch*head).
// ---------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads) fwd_f32_kernel(KArgs a) {
  constexpr int BM = 64, LD = D + 4, DV = D / 64;
  __shared__ float Qs[BM * LD];
  __shared__ float Ks[BN * LD];
  __shared__ float Vs[BN * LD];
  __shared__ float Ss[BM * SLD];
  __shared__ float row_m[BM], row_l[BM], row_alpha[BM];

  const int qt = blockIdx.x, g = blockIdx.y;
  const int b = blockIdx.z / a.H, h = blockIdx.z % a.H;
  const int c = h / a.r;
  const int s = shift_of_head(a, h);
  const int split = split_of_group(a, g, s);
  const int i0 = qt * BM;
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  const float* q = static_cast<const float*>(a.q);
  const float* k = static_cast<const float*>(a.k);
  const float* v = static_cast<const float*>(a.v);

  load_tile<BM, D>(Qs, q, a.sq, b, h, g, i0, s, a.N, a.G);
  if (tid < BM) { row_m[tid] = -1e30f; row_l[tid] = 0.f; }
  float o[4][DV][4];
#pragma unroll
  for (int x = 0; x < 4; ++x)
#pragma unroll
    for (int e = 0; e < DV; ++e)
#pragma unroll
      for (int y = 0; y < 4; ++y) o[x][e][y] = 0.f;

  const int jt_first = (i0 >= split ? split : 0) / BN;
  for (int jt = jt_first; jt <= qt; ++jt) {
    const int j0 = jt * BN;
    __syncthreads();
    load_tile<BN, D>(Ks, k, a.sk, b, c, g, j0, s, a.N, a.G);
    load_tile<BN, D>(Vs, v, a.sv, b, c, g, j0, s, a.N, a.G);
    __syncthreads();
    float acc[4][4];
    tile_nt<4, D>(acc, Qs, Ks, ty, tx);
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        int i = i0 + ty + 16 * x, j = j0 + tx + 16 * y;
        int lo = i >= split ? split : 0;
        bool vis = (j <= i) && (j >= lo);
        Ss[(ty + 16 * x) * SLD + tx + 16 * y] = vis ? acc[x][y] * a.scale_log2 : -INFINITY;
      }
    __syncthreads();
    {  // online softmax: 4 threads per row
      int row = tid / 4, part = tid % 4;
      float mx = -INFINITY;
#pragma unroll
      for (int x = 0; x < 16; ++x) mx = fmaxf(mx, Ss[row * SLD + part + 4 * x]);
      mx = fmaxf(mx, __shfl_xor(mx, 1));
      mx = fmaxf(mx, __shfl_xor(mx, 2));
      float m_old = row_m[row];
      float m_new = fmaxf(m_old, mx);
      float sum = 0.f;
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        float p = exp2f(Ss[row * SLD + part + 4 * x] - m_new);
        Ss[row * SLD + part + 4 * x] = p;
        sum += p;
      }
      sum += __shfl_xor(sum, 1);
      sum += __shfl_xor(sum, 2);
      if (part == 0) {
        float alpha = exp2f(m_old - m_new);
        row_alpha[row] = alpha;
        row_l[row] = row_l[row] * alpha + sum;
        row_m[row] = m_new;
      }
    }
    __syncthreads();
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      float al = row_alpha[ty + 16 * x];
#pragma unroll
      for (int e = 0; e < DV; ++e)
#pragma unroll
        for (int y = 0; y < 4; ++y) o[x][e][y] *= al;
    }
    for (int j = 0; j < BN; ++j) {
      float4 vv[DV];
#pragma unroll
      for (int e = 0; e < DV; ++e) vv[e] = *reinterpret_cast<const float4*>(Vs + j * LD + 4 * tx + 64 * e);
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        float p = Ss[(ty + 16 * x) * SLD + j];
#pragma unroll
        for (int e = 0; e < DV; ++e) {
          o[x][e][0] += p * vv[e].x; o[x][e][1] += p * vv[e].y;
          o[x][e][2] += p * vv[e].z; o[x][e][3] += p * vv[e].w;
        }
      }
    }
  }
  __syncthreads();
  float* out = static_cast<float*>(a.o);
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    int row = ty + 16 * x, i = i0 + row;
    if (i >= a.G) continue;
    int tok = token_of(g * a.G + i, s, a.N);
    float inv = 1.f / row_l[row];
#pragma unroll
    for (int e = 0; e < DV; ++e) {
      float4 val = make_float4(o[x][e][0] * inv, o[x][e][1] * inv, o[x][e][2] * inv, o[x][e][3] * inv);
      *reinterpret_cast<float4*>(out + row_off(a.so, b, tok, h) + 4 * tx + 64 * e) = val;
    }
    if (tx == 0)
      a.lse[((size_t)b * a.H + h) * a.N + tok] = (row_m[row] + log2f(row_l[row])) * 0.6931471805599453f;
  }
}

// ---------------------------------------------------------------------------
// dK/dV: one block per (key tile of 64 rows, group, batch * kv head * class).
// Loops over the query heads of the kv head that belong to the class (shifted or
// not) and over query tiles at or below the diagonal.
// ---------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads) bwd_dkdv_f32_kernel(KArgs a, int ncls) {
  constexpr int BQ = 32, LD = D + 4, DV = D / 64;
  __shared__ float Ks[BN * LD];
  __shared__ float Vs[BN * LD];
  __shared__ float Qs[BQ * LD];
  __shared__ float dOs[BQ * LD];
  __shared__ float Ps[BQ * SLD];
  __shared__ float dSs[BQ * SLD];
  __shared__ float row_lse[BQ], row_delta[BQ];

  const int jt = blockIdx.x, g = blockIdx.y;
  int z = blockIdx.z;
  const int cls_slot = z % ncls; z /= ncls;
  const int c = z % a.Hkv, b = z / a.Hkv;
  // head range of this kv head in this class
  int h_lo = c * a.r, h_hi = (c + 1) * a.r;
  int cls;
  if (ncls == 2) {
    cls = cls_slot;
  } else {
    cls = h_lo >= a.shifted_from ? 1 : 0;   // unmixed: every head of c is in one class
  }
  if (cls == 0) h_hi = min(h_hi, a.shifted_from); else h_lo = max(h_lo, a.shifted_from);
  // (an empty class still writes its zero partial so that the combine pass can sum both)
  const int s = cls ? a.shift : 0;
  const int split = split_of_group(a, g, s);
  const int j0 = jt * BN;
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  const float* q = static_cast<const float*>(a.q);
  const float* k = static_cast<const float*>(a.k);
  const float* v = static_cast<const float*>(a.v);
  const float* dout = static_cast<const float*>(a.dout);

  load_tile<BN, D>(Ks, k, a.sk, b, c, g, j0, s, a.N, a.G);
  load_tile<BN, D>(Vs, v, a.sv, b, c, g, j0, s, a.N, a.G);
  float dk[4][DV][4], dv[4][DV][4];
#pragma unroll
  for (int x = 0; x < 4; ++x)
#pragma unroll
    for (int e = 0; e < DV; ++e)
#pragma unroll
      for (int y = 0; y < 4; ++y) { dk[x][e][y] = 0.f; dv[x][e][y] = 0.f; }

  const int n_qt = (a.G + BQ - 1) / BQ;
  for (int h = h_lo; h < h_hi; ++h) {
    for (int it = j0 / BQ; it < n_qt; ++it) {
      const int i0 = it * BQ;
      if (j0 + BN - 1 < split && i0 >= split) break;   // Variant 2: keys of the first block see no later rows
      __syncthreads();
      load_tile<BQ, D>(Qs, q, a.sq, b, h, g, i0, s, a.N, a.G);
      load_tile<BQ, D>(dOs, dout, a.so, b, h, g, i0, s, a.N, a.G);
      if (tid < BQ) {
        int i = i0 + tid;
        float l = 0.f, dl = 0.f;
        if (i < a.G) {
          int tok = token_of(g * a.G + i, s, a.N);
          l = a.lse[((size_t)b * a.H + h) * a.N + tok];
          dl = a.delta[((size_t)b * a.H + h) * a.N + tok];
        }
        row_lse[tid] = l * 1.4426950408889634f;
        row_delta[tid] = dl;
      }
      __syncthreads();
      float sacc[2][4], pacc[2][4];
      tile_nt<2, D>(sacc, Qs, Ks, ty, tx);
      tile_nt<2, D>(pacc, dOs, Vs, ty, tx);
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) {
          int row = ty + 16 * x, col = tx + 16 * y;
          int i = i0 + row, j = j0 + col;
          int lo = i >= split ? split : 0;
          bool vis = (j <= i) && (j >= lo) && (i < a.G);
          float p = vis ? exp2f(sacc[x][y] * a.scale_log2 - row_lse[row]) : 0.f;
          Ps[row * SLD + col] = p;
          dSs[row * SLD + col] = p * (pacc[x][y] - row_delta[row]);
        }
      __syncthreads();
      for (int i = 0; i < BQ; ++i) {
        float4 dov[DV], qv[DV];
#pragma unroll
        for (int e = 0; e < DV; ++e) {
          dov[e] = *reinterpret_cast<const float4*>(dOs + i * LD + 4 * tx + 64 * e);
          qv[e] = *reinterpret_cast<const float4*>(Qs + i * LD + 4 * tx + 64 * e);
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          float p = Ps[i * SLD + ty + 16 * x];
          float ds = dSs[i * SLD + ty + 16 * x];
#pragma unroll
          for (int e = 0; e < DV; ++e) {
            dv[x][e][0] += p * dov[e].x; dv[x][e][1] += p * dov[e].y;
            dv[x][e][2] += p * dov[e].z; dv[x][e][3] += p * dov[e].w;
            dk[x][e][0] += ds * qv[e].x; dk[x][e][1] += ds * qv[e].y;
            dk[x][e][2] += ds * qv[e].z; dk[x][e][3] += ds * qv[e].w;
          }
        }
      }
    }
  }
  // store: directly, or as an fp32 partial of this class when kv heads are mixed
  const size_t kv_elems = (size_t)a.B * a.N * a.Hkv * D;
  float* dk_out = a.dkv_partial ? a.dkv_partial + (size_t)cls * kv_elems : static_cast<float*>(a.dk);
  float* dv_out = a.dkv_partial ? a.dkv_partial + (size_t)(2 + cls) * kv_elems : static_cast<float*>(a.dv);
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    int j = j0 + ty + 16 * x;
    if (j >= a.G) continue;
    int tok = token_of(g * a.G + j, s, a.N);
    // fp32 partials of a mixed kv head are contiguous; final dk, dv may be strided views
    const size_t cont = ((size_t)((size_t)b * a.N + tok) * a.Hkv + c) * D + 4 * tx;
    const size_t base = a.dkv_partial ? cont : row_off(a.sdk, b, tok, c) + 4 * tx;
    const size_t base_v = a.dkv_partial ? cont : row_off(a.sdv, b, tok, c) + 4 * tx;
#pragma unroll
    for (int e = 0; e < DV; ++e) {
      *reinterpret_cast<float4*>(dk_out + base + 64 * e) =
          make_float4(dk[x][e][0] * a.scale, dk[x][e][1] * a.scale, dk[x][e][2] * a.scale, dk[x][e][3] * a.scale);
      *reinterpret_cast<float4*>(dv_out + base_v + 64 * e) =
          make_float4(dv[x][e][0], dv[x][e][1], dv[x][e][2], dv[x][e][3]);
    }
  }
}

// ---------------------------------------------------------------------------
// dQ: one block per (query tile of 32 rows, group, batch*head).
// ---------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads) bwd_dq_f32_kernel(KArgs a) {
  constexpr int BQ = 32, LD = D + 4, DV = D / 64;
  __shared__ float Ks[BN * LD];
  __shared__ float Vs[BN * LD];
  __shared__ float Qs[BQ * LD];
  __shared__ float dOs[BQ * LD];
  __shared__ float dSs[BQ * SLD];
  __shared__ float row_lse[BQ], row_delta[BQ];

  const int qt = blockIdx.x, g = blockIdx.y;
  const int b = blockIdx.z / a.H, h = blockIdx.z % a.H;
  const int c = h / a.r;
  const int s = shift_of_head(a, h);
  const int split = split_of_group(a, g, s);
  const int i0 = qt * BQ;
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  const float* q = static_cast<const float*>(a.q);
  const float* k = static_cast<const float*>(a.k);
  const float* v = static_cast<const float*>(a.v);
  const float* dout = static_cast<const float*>(a.dout);

  load_tile<BQ, D>(Qs, q, a.sq, b, h, g, i0, s, a.N, a.G);
  load_tile<BQ, D>(dOs, dout, a.so, b, h, g, i0, s, a.N, a.G);
  if (tid < BQ) {
    int i = i0 + tid;
    float l = 0.f, dl = 0.f;
    if (i < a.G) {
      int tok = token_of(g * a.G + i, s, a.N);
      l = a.lse[((size_t)b * a.H + h) * a.N + tok];
      dl = a.delta[((size_t)b * a.H + h) * a.N + tok];
    }
    row_lse[tid] = l * 1.4426950408889634f;
    row_delta[tid] = dl;
  }
  float dq[2][DV][4];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int e = 0; e < DV; ++e)
#pragma unroll
      for (int y = 0; y < 4; ++y) dq[x][e][y] = 0.f;

  const int jt_first = (i0 >= split ? split : 0) / BN;
  const int jt_last = min(i0 + BQ - 1, a.G - 1) / BN;
  for (int jt = jt_first; jt <= jt_last; ++jt) {
    const int j0 = jt * BN;
    __syncthreads();
    load_tile<BN, D>(Ks, k, a.sk, b, c, g, j0, s, a.N, a.G);
    load_tile<BN, D>(Vs, v, a.sv, b, c, g, j0, s, a.N, a.G);
    __syncthreads();
    float sacc[2][4], pacc[2][4];
    tile_nt<2, D>(sacc, Qs, Ks, ty, tx);
    tile_nt<2, D>(pacc, dOs, Vs, ty, tx);
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        int row = ty + 16 * x, col = tx + 16 * y;
        int i = i0 + row, j = j0 + col;
        int lo = i >= split ? split : 0;
        bool vis = (j <= i) && (j >= lo) && (i < a.G);
        float p = vis ? exp2f(sacc[x][y] * a.scale_log2 - row_lse[row]) : 0.f;
        dSs[row * SLD + col] = p * (pacc[x][y] - row_delta[row]);
      }
    __syncthreads();
    for (int j = 0; j < BN; ++j) {
      float4 kv[DV];
#pragma unroll
      for (int e = 0; e < DV; ++e) kv[e] = *reinterpret_cast<const float4*>(Ks + j * LD + 4 * tx + 64 * e);
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        float ds = dSs[(ty + 16 * x) * SLD + j];
#pragma unroll
        for (int e = 0; e < DV; ++e) {
          dq[x][e][0] += ds * kv[e].x; dq[x][e][1] += ds * kv[e].y;
          dq[x][e][2] += ds * kv[e].z; dq[x][e][3] += ds * kv[e].w;
        }
      }
    }
  }
  float* out = static_cast<float*>(a.dq);
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    int i = i0 + ty + 16 * x;
    if (i >= a.G) continue;
    int tok = token_of(g * a.G + i, s, a.N);
#pragma unroll
    for (int e = 0; e < DV; ++e)
      *reinterpret_cast<float4*>(out + row_off(a.sdq, b, tok, h) + 4 * tx + 64 * e) =
          make_float4(dq[x][e][0] * a.scale, dq[x][e][1] * a.scale, dq[x][e][2] * a.scale, dq[x][e][3] * a.scale);
  }
}

template <int D>
int launch_fwd_t(const KArgs& a, hipStream_t st) {
  dim3 grid((a.G + 63) / 64, a.N / a.G, a.B * a.H);
  hipLaunchKernelGGL(fwd_f32_kernel<D>, grid, dim3(kThreads), 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int D>
int launch_dkdv_t(const KArgs& a, hipStream_t st) {
  const int ncls = a.mixed ? 2 : 1;
  dim3 g1((a.G + 63) / 64, a.N / a.G, a.B * a.Hkv * ncls);
  hipLaunchKernelGGL(bwd_dkdv_f32_kernel<D>, g1, dim3(kThreads), 0, st, a, ncls);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int D>
int launch_dq_t(const KArgs& a, hipStream_t st) {
  dim3 g2((a.G + 31) / 32, a.N / a.G, a.B * a.H);
  hipLaunchKernelGGL(bwd_dq_f32_kernel<D>, g2, dim3(kThreads), 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace

int launch_fwd_f32(const KArgs& a, hipStream_t st) {
  return a.D == 64 ? launch_fwd_t<64>(a, st) : launch_fwd_t<128>(a, st);
}

int launch_bwd_dkdv_f32(const KArgs& a, hipStream_t st) {
  return a.D == 64 ? launch_dkdv_t<64>(a, st) : launch_dkdv_t<128>(a, st);
}

int launch_bwd_dq_f32(const KArgs& a, hipStream_t st) {
  return a.D == 64 ? launch_dq_t<64>(a, st) : launch_dq_t<128>(a, st);
}

}  // namespace s2
