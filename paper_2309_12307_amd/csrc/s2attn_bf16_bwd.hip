// bf16 S2-Attn backward for gfx950: dK/dV kernel and dQ kernel.  Both recompute
// P = exp(scale*S - lse) from the stored log-sum-exp and use the softmax-Jacobian
// form dS = P * (dP - delta), delta_i = dO_i . O_i (computed by the pre-pass).
// The shift/group map of LongLoRA Algorithm 1 is row addressing only.
//
// dK/dV: a workgroup owns 128 keys of one (batch, kv head, class, group); a wave owns
//   32 of them with their K^T and V^T fragments in registers.  It walks the query
//   tiles (64 rows, staged in LDS) at or below the diagonal for every query head of
//   the kv head.  S = Q K^T and dP = dO V^T come out with keys lane-indexed and
//   queries register-indexed, so P and dS feed dV^T += dO^T P and dK^T += Q^T dS as
//   B operands unchanged, with dO^T and Q^T read through transposing LDS loads.
// dQ: a workgroup owns 128 query rows (32 per wave, Q^T and dO^T fragments in
//   registers) and walks the 64-key tiles up to the diagonal: S^T = K Q^T,
//   dP^T = V dO^T, dQ^T += K^T dS^T with K^T through transposing LDS loads.
#include "s2attn_bf16_common.h"
#include "s2attn_device.h"
#include "s2attn_launch.h"

namespace s2 {
namespace {

constexpr int kTileRows = 64;
constexpr int kTileBytes = kTileRows * kRowBytes;   // 16 KB

// Transposes a wave's 32 x 128 accumulator block (rows lane-indexed, columns
// register-indexed) through its private 8 KB LDS region.
__device__ __forceinline__ void acc_to_lds(char* region, const f32x16 (&acc)[4], float mul, int l32, int g32) {
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) {
      const bf16x4 pk = pack4(acc[db][4 * vv] * mul, acc[db][4 * vv + 1] * mul,
                              acc[db][4 * vv + 2] * mul, acc[db][4 * vv + 3] * mul);
      *reinterpret_cast<bf16x4*>(region + tile_off(l32, 4 * db + vv) + 8 * g32) = pk;
    }
}

// ---------------------------------------------------------------------------
// dK / dV
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256, 1)
bwd_dkdv_bf16_kernel(KArgs a, int ncls, int T, int n_rest) {
  __shared__ __attribute__((aligned(16))) char smem[4 * kTileBytes];   // [stage][Q,dO]
  __shared__ __attribute__((aligned(16))) float rows_s[2][2][kTileRows];                          // [stage][lse*log2e, delta]

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int g32 = lane >> 5, l32 = lane & 31;

  // block -> (batch, kv head, class, group, key tile); heaviest key tiles (jt = 0) first
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int y = slot / T;
  const int jt = slot - y * T;
  int rest = y * 8 + xcd;
  if (rest >= n_rest) return;
  const int NG = a.N / a.G;
  const int gidx = rest % NG; rest /= NG;
  const int cls_slot = rest % ncls; rest /= ncls;
  const int c = rest % a.Hkv;
  const int b = rest / a.Hkv;

  int h_lo = c * a.r, h_hi = (c + 1) * a.r;
  const int cls = ncls == 2 ? cls_slot : (h_lo >= a.shifted_from ? 1 : 0);
  if (cls == 0) h_hi = min(h_hi, a.shifted_from); else h_lo = max(h_lo, a.shifted_from);
  const int nheads = max(h_hi - h_lo, 0);

  const int s = cls ? a.shift : 0;
  const int split = split_of_group(a, gidx, s);
  const int j0 = jt * 128;
  const int kw0 = j0 + 32 * w;                       // first key of this wave
  const int it_begin = j0 / kTileRows;
  const int it_end = (j0 + 127 < split ? split : a.G) / kTileRows;
  const int nq = it_end - it_begin;
  const int n_iter = nheads * nq;
  const float c2 = a.scale_log2;

  const __bf16* qp = static_cast<const __bf16*>(a.q);
  const __bf16* kp = static_cast<const __bf16*>(a.k);
  const __bf16* vp = static_cast<const __bf16*>(a.v);
  const __bf16* dop = static_cast<const __bf16*>(a.dout);

  // K^T and V^T fragments of this wave's 32 keys
  bf16x8 kf[8], vf[8];
  {
    const int tok = token_of(gidx * a.G + kw0 + l32, s, a.N);
    const size_t off = ((size_t)((size_t)b * a.N + tok) * a.Hkv + c) * 128;
    const bf16x8* ksrc = reinterpret_cast<const bf16x8*>(kp + off);
    const bf16x8* vsrc = reinterpret_cast<const bf16x8*>(vp + off);
#pragma unroll
    for (int st = 0; st < 8; ++st) { kf[st] = ksrc[2 * st + g32]; vf[st] = vsrc[2 * st + g32]; }
  }

  const int ld_row = tid >> 4, ld_chunk = tid & 15;
  uint4 qreg[4], doreg[4];
  float rowreg = 0.f;
  auto issue_loads = [&](int n) {
    const int h = h_lo + n / nq;
    const int it = it_begin + n % nq;
    const int tok0 = token_of(gidx * a.G + it * kTileRows, s, a.N);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const size_t off = ((size_t)((size_t)b * a.N + tok0 + ld_row + 16 * p) * a.H + h) * 128 + ld_chunk * 8;
      qreg[p] = *reinterpret_cast<const uint4*>(qp + off);
      doreg[p] = *reinterpret_cast<const uint4*>(dop + off);
    }
    if (tid < 128) {
      const size_t ro = ((size_t)b * a.H + h) * a.N + tok0 + (tid & 63);
      rowreg = tid < 64 ? a.lse[ro] * kLog2e : a.delta[ro];
    }
  };
  auto store_lds = [&](int stage) {
    char* Qs = smem + stage * 2 * kTileBytes;
    char* dOs = Qs + kTileBytes;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int off = tile_off(ld_row + 16 * p, ld_chunk);
      *reinterpret_cast<uint4*>(Qs + off) = qreg[p];
      *reinterpret_cast<uint4*>(dOs + off) = doreg[p];
    }
    if (tid < 128) rows_s[stage][tid >> 6][tid & 63] = rowreg;
  };

  f32x16 dk_acc[4], dv_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) { dk_acc[db] = zero16(); dv_acc[db] = zero16(); }

  if (n_iter > 0) {
    issue_loads(0);
    store_lds(0);
  }
  __syncthreads();

  for (int n = 0; n < n_iter; ++n) {
    const int stage = n & 1;
    const bool has_next = n + 1 < n_iter;
    if (has_next) issue_loads(n + 1);
    const int q0 = (it_begin + n % nq) * kTileRows;
    // work for this wave: some query at or after its first key, and (Variant 2) not a
    // query tile of the second block when the wave's keys are in the first block
    if (q0 + kTileRows - 1 >= kw0 && !(kw0 + 31 < split && q0 >= split)) {
      const char* Qs = smem + stage * 2 * kTileBytes;
      const char* dOs = Qs + kTileBytes;
      bf16x8 pf[2][2], dsf[2][2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        f32x16 s_acc = zero16(), dp_acc = zero16();
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          s_acc = mfma32(frag_rm(Qs, 32 * mb + l32, 2 * st + g32), kf[st], s_acc);
          dp_acc = mfma32(frag_rm(dOs, 32 * mb + l32, 2 * st + g32), vf[st], dp_acc);
        }
        const bool diag = q0 + 32 * mb < kw0 + 31;    // some query of this block precedes some key
        const int key = kw0 + l32;
        float p[16], ds[16];
#pragma unroll
        for (int vv = 0; vv < 4; ++vv) {
          const float4 l4 = *reinterpret_cast<const float4*>(&rows_s[stage][0][32 * mb + 8 * vv + 4 * g32]);
          const float4 d4 = *reinterpret_cast<const float4*>(&rows_s[stage][1][32 * mb + 8 * vv + 4 * g32]);
          const float ls[4] = {l4.x, l4.y, l4.z, l4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int v = 4 * vv + e;
            float pv = __builtin_amdgcn_exp2f(fmaf(s_acc[v], c2, -ls[e]));
            if (diag) {
              const int qrow = q0 + 32 * mb + 8 * vv + 4 * g32 + e;
              if (key > qrow) pv = 0.f;
            }
            p[v] = pv;
            ds[v] = pv * (dp_acc[v] - dl[e]);
          }
        }
        pf[mb][0] = pack8(p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]);
        pf[mb][1] = pack8(p[8], p[9], p[10], p[11], p[12], p[13], p[14], p[15]);
        dsf[mb][0] = pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
        dsf[mb][1] = pack8(ds[8], ds[9], ds[10], ds[11], ds[12], ds[13], ds[14], ds[15]);
      }
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int db = 0; db < 4; ++db) {
            dv_acc[db] = mfma32(frag_tr(dOs, 32 * mb + 16 * t, db, lane), pf[mb][t], dv_acc[db]);
            dk_acc[db] = mfma32(frag_tr(Qs, 32 * mb + 16 * t, db, lane), dsf[mb][t], dk_acc[db]);
          }
    }
    if (has_next) store_lds(stage ^ 1);
    __syncthreads();
  }

  // ---- store dK^T, dV^T blocks (keys lane-indexed) at un-rolled token rows
  if (a.dkv_partial) {
    // kv head shared by both classes: fp32 partial of this class, summed by the combine pass
    const size_t kv_elems = (size_t)a.B * a.N * a.Hkv * 128;
    float* dk_out = a.dkv_partial + (size_t)cls * kv_elems;
    float* dv_out = a.dkv_partial + (size_t)(2 + cls) * kv_elems;
    const int tok = token_of(gidx * a.G + kw0 + l32, s, a.N);
    const size_t base = ((size_t)((size_t)b * a.N + tok) * a.Hkv + c) * 128;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) {
        const int d = 32 * db + 8 * vv + 4 * g32;
        *reinterpret_cast<float4*>(dk_out + base + d) =
            make_float4(dk_acc[db][4 * vv] * a.scale, dk_acc[db][4 * vv + 1] * a.scale,
                        dk_acc[db][4 * vv + 2] * a.scale, dk_acc[db][4 * vv + 3] * a.scale);
        *reinterpret_cast<float4*>(dv_out + base + d) =
            make_float4(dv_acc[db][4 * vv], dv_acc[db][4 * vv + 1], dv_acc[db][4 * vv + 2], dv_acc[db][4 * vv + 3]);
      }
    return;
  }
  char* rk = smem + w * (32 * kRowBytes);
  char* rv = smem + (4 + w) * (32 * kRowBytes);
  acc_to_lds(rk, dk_acc, a.scale, l32, g32);
  acc_to_lds(rv, dv_acc, 1.f, l32, g32);
  __syncthreads();
  __bf16* dkp = static_cast<__bf16*>(a.dk);
  __bf16* dvp = static_cast<__bf16*>(a.dv);
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int row = it * 4 + (lane >> 4), ch = lane & 15;
    const int tok = token_of(gidx * a.G + kw0 + row, s, a.N);
    const size_t off = ((size_t)((size_t)b * a.N + tok) * a.Hkv + c) * 128 + ch * 8;
    *reinterpret_cast<uint4*>(dkp + off) = *reinterpret_cast<const uint4*>(rk + tile_off(row, ch));
    *reinterpret_cast<uint4*>(dvp + off) = *reinterpret_cast<const uint4*>(rv + tile_off(row, ch));
  }
}

// ---------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256, 2)
bwd_dq_bf16_kernel(KArgs a, int T, int n_rest) {
  constexpr int BM = 128, BN = 64;
  __shared__ __attribute__((aligned(16))) char smem[4 * kTileBytes];   // [stage][K,V]

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int g32 = lane >> 5, l32 = lane & 31;

  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int y = slot / T;
  const int qt = T - 1 - (slot - y * T);
  const int hr = y % a.r;
  int rest = (y / a.r) * 8 + xcd;
  if (rest >= n_rest) return;
  const int NG = a.N / a.G;
  const int gidx = rest % NG; rest /= NG;
  const int c = rest % a.Hkv;
  const int b = rest / a.Hkv;
  const int h = c * a.r + hr;

  const int s = shift_of_head(a, h);
  const int split = split_of_group(a, gidx, s);
  const int i0 = qt * BM;
  const int qw0 = i0 + w * 32;
  const int lo_w = qw0 >= split ? split : 0;
  const int jt_first = (i0 >= split ? split : 0) / BN;
  const int jt_last = (i0 + BM - 1) / BN;
  const float c2 = a.scale_log2;

  const __bf16* qp = static_cast<const __bf16*>(a.q);
  const __bf16* kp = static_cast<const __bf16*>(a.k);
  const __bf16* vp = static_cast<const __bf16*>(a.v);
  const __bf16* dop = static_cast<const __bf16*>(a.dout);

  bf16x8 qf[8], dof[8];
  float lse2, delta;
  {
    const int tok = token_of(gidx * a.G + qw0 + l32, s, a.N);
    const size_t off = ((size_t)((size_t)b * a.N + tok) * a.H + h) * 128;
    const bf16x8* qsrc = reinterpret_cast<const bf16x8*>(qp + off);
    const bf16x8* dsrc = reinterpret_cast<const bf16x8*>(dop + off);
#pragma unroll
    for (int st = 0; st < 8; ++st) { qf[st] = qsrc[2 * st + g32]; dof[st] = dsrc[2 * st + g32]; }
    const size_t ro = ((size_t)b * a.H + h) * a.N + tok;
    lse2 = a.lse[ro] * kLog2e;
    delta = a.delta[ro];
  }

  const int ld_row = tid >> 4, ld_chunk = tid & 15;
  uint4 kreg[4], vreg[4];
  auto issue_loads = [&](int jt) {
    const int tok0 = token_of(gidx * a.G + jt * BN, s, a.N);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const size_t off = ((size_t)((size_t)b * a.N + tok0 + ld_row + 16 * p) * a.Hkv + c) * 128 + ld_chunk * 8;
      kreg[p] = *reinterpret_cast<const uint4*>(kp + off);
      vreg[p] = *reinterpret_cast<const uint4*>(vp + off);
    }
  };
  auto store_lds = [&](int stage) {
    char* Ks = smem + stage * 2 * kTileBytes;
    char* Vs = Ks + kTileBytes;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int off = tile_off(ld_row + 16 * p, ld_chunk);
      *reinterpret_cast<uint4*>(Ks + off) = kreg[p];
      *reinterpret_cast<uint4*>(Vs + off) = vreg[p];
    }
  };

  f32x16 dq_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) dq_acc[db] = zero16();

  issue_loads(jt_first);
  store_lds(0);
  __syncthreads();

  for (int jt = jt_first; jt <= jt_last; ++jt) {
    const int stage = (jt - jt_first) & 1;
    const bool has_next = jt < jt_last;
    if (has_next) issue_loads(jt + 1);
    const int j0 = jt * BN;
    const bool active = (j0 <= qw0 + 31) && (j0 + BN - 1 >= lo_w);
    if (active) {
      const char* Ks = smem + stage * 2 * kTileBytes;
      const char* Vs = Ks + kTileBytes;
      bf16x8 dsf[2][2];
      const bool diag = j0 + BN - 1 > qw0;
      const int qrow = qw0 + l32;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        f32x16 s_acc = zero16(), dp_acc = zero16();
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          s_acc = mfma32(frag_rm(Ks, 32 * mb + l32, 2 * st + g32), qf[st], s_acc);
          dp_acc = mfma32(frag_rm(Vs, 32 * mb + l32, 2 * st + g32), dof[st], dp_acc);
        }
        float ds[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float pv = __builtin_amdgcn_exp2f(fmaf(s_acc[v], c2, -lse2));
          if (diag) {
            const int key = j0 + 32 * mb + 8 * (v >> 2) + 4 * g32 + (v & 3);
            if (key > qrow) pv = 0.f;
          }
          ds[v] = pv * (dp_acc[v] - delta);
        }
        dsf[mb][0] = pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
        dsf[mb][1] = pack8(ds[8], ds[9], ds[10], ds[11], ds[12], ds[13], ds[14], ds[15]);
      }
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int db = 0; db < 4; ++db)
            dq_acc[db] = mfma32(frag_tr(Ks, 32 * mb + 16 * t, db, lane), dsf[mb][t], dq_acc[db]);
    }
    if (has_next) store_lds(stage ^ 1);
    __syncthreads();
  }

  char* region = smem + w * (32 * kRowBytes);
  acc_to_lds(region, dq_acc, a.scale, l32, g32);
  __syncthreads();
  __bf16* dqp = static_cast<__bf16*>(a.dq);
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int row = it * 4 + (lane >> 4), ch = lane & 15;
    const int tok = token_of(gidx * a.G + qw0 + row, s, a.N);
    *reinterpret_cast<uint4*>(dqp + ((size_t)((size_t)b * a.N + tok) * a.H + h) * 128 + ch * 8) =
        *reinterpret_cast<const uint4*>(region + tile_off(row, ch));
  }
}

}  // namespace

int launch_bwd_dkdv_bf16(const KArgs& a, hipStream_t st) {
  const int NG = a.N / a.G;
  const int ncls = a.mixed ? 2 : 1;
  const int T = a.G / 128;
  const int n_rest = a.B * a.Hkv * ncls * NG;
  const int blocks = 8 * T * ((n_rest + 7) / 8);
  hipLaunchKernelGGL(bwd_dkdv_bf16_kernel, dim3(blocks), dim3(256), 0, st, a, ncls, T, n_rest);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_bwd_dq_bf16(const KArgs& a, hipStream_t st) {
  const int NG = a.N / a.G;
  const int T = a.G / 128;
  const int n_rest = a.B * a.Hkv * NG;
  const int blocks = 8 * T * a.r * ((n_rest + 7) / 8);
  hipLaunchKernelGGL(bwd_dq_bf16_kernel, dim3(blocks), dim3(256), 0, st, a, T, n_rest);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace s2
