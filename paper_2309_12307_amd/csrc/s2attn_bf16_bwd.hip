// bf16 S2-Attn backward for gfx950: dK/dV kernel and dQ kernel.  Both recompute
// P = exp(scale*S - lse) from the stored log-sum-exp and use the softmax-Jacobian
// form dS = P * (dP - delta), delta_i = dO_i . O_i (computed by the pre-pass).
// The shift/group map of LongLoRA Algorithm 1 is row addressing only.
//
// dK/dV: a workgroup owns 128 keys of one (batch, kv head, class, group); a wave owns
//   32 of them with their K^T and V^T fragments in registers.  It walks the 128-row
//   query tiles (staged in LDS by direct global->LDS loads, two stages) at or below
//   the diagonal for every query head of the kv head.  S = Q K^T and dP = dO V^T come
//   out with keys lane-indexed and queries register-indexed, so P and dS feed
//   dV^T += dO^T P and dK^T += Q^T dS as B operands unchanged, with dO^T and Q^T read
//   through transposing LDS loads.  One wave per SIMD: the 32-query blocks of a tile
//   are software-pipelined so that the VALU work of one block sits between the MFMAs
//   of its neighbours.
// dQ: a workgroup owns 128 query rows (32 per wave, Q^T and dO^T fragments in
//   registers) and walks the 64-key tiles up to the diagonal: S^T = K Q^T,
//   dP^T = V dO^T, dQ^T += K^T dS^T with K^T through transposing LDS loads.
#include "s2attn_bf16_common.h"
#include "s2attn_device.h"
#include "s2attn_launch.h"

namespace s2 {
namespace {

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

// ===========================================================================
// dK / dV
// ===========================================================================
constexpr int kQTileRows = 128;
constexpr int kQTileBytes = kQTileRows * kRowBytes;   // 32 KB

struct DkdvBlock {     // S and dP accumulators of one 32-query block
  f32x16 s, dp;
};

// S = Q K^T and dP = dO V^T for query block mb of the staged tile.
__device__ __forceinline__ void dkdv_scores(DkdvBlock& blk, const char* Qs, const char* dOs, int mb,
                                            const bf16x8 (&kf)[8], const bf16x8 (&vf)[8], int l32, int g32) {
  blk.s = zero16();
  blk.dp = zero16();
  bf16x8 qa[4], da[4];
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      qa[i] = frag_rm(Qs, 32 * mb + l32, 2 * (4 * half + i) + g32);
      da[i] = frag_rm(dOs, 32 * mb + l32, 2 * (4 * half + i) + g32);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      blk.s = mfma32(qa[i], kf[4 * half + i], blk.s);
      blk.dp = mfma32(da[i], vf[4 * half + i], blk.dp);
    }
  }
}

// P and dS of a block as packed bf16 B operands (two 16-query k-steps each).
template <bool MASK>
__device__ __forceinline__ void dkdv_softmax(const DkdvBlock& blk, const float* lse_s, const float* delta_s, int mb,
                                             int q_first, int key, float c2, int g32,
                                             bf16x8 (&pf)[2], bf16x8 (&dsf)[2]) {
  float p[16], ds[16];
#pragma unroll
  for (int vv = 0; vv < 4; ++vv) {
    const float4 l4 = *reinterpret_cast<const float4*>(lse_s + 32 * mb + 8 * vv + 4 * g32);
    const float4 d4 = *reinterpret_cast<const float4*>(delta_s + 32 * mb + 8 * vv + 4 * g32);
    const float ls[4] = {l4.x, l4.y, l4.z, l4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int v = 4 * vv + e;
      float pv = __builtin_amdgcn_exp2f(fmaf(blk.s[v], c2, -ls[e] * kLog2e));
      if (MASK) {
        const int qrow = q_first + 8 * vv + 4 * g32 + e;
        if (key > qrow) pv = 0.f;
      }
      p[v] = pv;
      ds[v] = pv * (blk.dp[v] - dl[e]);
    }
  }
  pf[0] = pack8(p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]);
  pf[1] = pack8(p[8], p[9], p[10], p[11], p[12], p[13], p[14], p[15]);
  dsf[0] = pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
  dsf[1] = pack8(ds[8], ds[9], ds[10], ds[11], ds[12], ds[13], ds[14], ds[15]);
}

// dV^T += dO^T P and dK^T += Q^T dS for query block mb.
__device__ __forceinline__ void dkdv_accumulate(f32x16 (&dk_acc)[4], f32x16 (&dv_acc)[4], const char* Qs,
                                                const char* dOs, int mb, const bf16x8 (&pf)[2],
                                                const bf16x8 (&dsf)[2], int lane) {
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    bf16x8 dot[4], qt[4];
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      dot[db] = frag_tr(dOs, 32 * mb + 16 * t, db, lane);
      qt[db] = frag_tr(Qs, 32 * mb + 16 * t, db, lane);
    }
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      dv_acc[db] = mfma32(dot[db], pf[t], dv_acc[db]);
      dk_acc[db] = mfma32(qt[db], dsf[t], dk_acc[db]);
    }
  }
}

__global__ void __launch_bounds__(256, 1)
bwd_dkdv_bf16_kernel(KArgs a, int ncls, int T, int n_rest) {
  __shared__ __attribute__((aligned(1024))) char smem[4 * kQTileBytes];            // [stage][Q,dO]
  __shared__ __attribute__((aligned(1024))) float rows_s[2][2][kQTileRows];        // [stage][lse, delta]

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
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
  const int key = kw0 + l32;
  // query rows visible to this workgroup's keys: [j0, q_end)
  const int q_end = (j0 + 127 < split) ? split : a.G;
  const int it_begin = j0 / kQTileRows;
  const int nq = (q_end - j0 + kQTileRows - 1) / kQTileRows;
  const int n_iter = nheads * nq;
  const float c2 = a.scale_log2;

  const char* qp = static_cast<const char*>(a.q);
  const char* dop = static_cast<const char*>(a.dout);

  // K^T and V^T fragments of this wave's 32 keys
  bf16x8 kf[8], vf[8];
  {
    const int tok = token_of(gidx * a.G + key, s, a.N);
    const size_t off = ((size_t)((size_t)b * a.N + tok) * a.Hkv + c) * 128;
    const bf16x8* ksrc = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(a.k) + off);
    const bf16x8* vsrc = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(a.v) + off);
#pragma unroll
    for (int st = 0; st < 8; ++st) { kf[st] = ksrc[2 * st + g32]; vf[st] = vsrc[2 * st + g32]; }
  }

  // staging: wave w, pass p fills tile rows 16p + 4w .. +3 (1 KB); every 64 rows of a
  // tile are one contiguous token run (shift and G are multiples of 64).
  const uint32_t smem_base = lds_addr(smem);
  const uint32_t rows_base = lds_addr(rows_s);
  const size_t q_row_bytes = (size_t)a.H * 256;
  const int st_row = 4 * w + (lane >> 4);
  const size_t st_goff = (size_t)st_row * q_row_bytes + (size_t)(((lane & 15) ^ swz(st_row)) << 4);
  auto issue_tile = [&](int n, int stage) {
    const int h = h_lo + n / nq;
    const int q0 = (it_begin + n % nq) * kQTileRows;
    const uint32_t qs = smem_base + stage * 2 * kQTileBytes + 4 * w * kRowBytes;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const int tok0 = token_of(gidx * a.G + q0 + 64 * hf, s, a.N);
      const size_t base = ((size_t)((size_t)b * a.N + tok0) * a.H + h) * 256;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const size_t go = base + st_goff + (size_t)p * 16 * q_row_bytes;
        dma16(qp + go, qs + (64 * hf + 16 * p) * kRowBytes);
        dma16(dop + go, qs + (64 * hf + 16 * p) * kRowBytes + kQTileBytes);
      }
      if (w == hf) {   // wave 0 / 1: lse and delta of rows 64*hf .. +63
        const size_t ro = ((size_t)b * a.H + h) * a.N + tok0 + lane;
        dma4(a.lse + ro, rows_base + ((stage * 2 + 0) * kQTileRows + 64 * hf) * 4);
        dma4(a.delta + ro, rows_base + ((stage * 2 + 1) * kQTileRows + 64 * hf) * 4);
      }
    }
  };

  f32x16 dk_acc[4], dv_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) { dk_acc[db] = zero16(); dv_acc[db] = zero16(); }

  if (n_iter > 0) issue_tile(0, 0);
  for (int n = 0; n < n_iter; ++n) {
    const int stage = n & 1;
    wait_vmcnt0();
    __syncthreads();
    if (n + 1 < n_iter) issue_tile(n + 1, stage ^ 1);
    const int q0 = (it_begin + n % nq) * kQTileRows;
    const char* Qs = smem + stage * 2 * kQTileBytes;
    const char* dOs = Qs + kQTileBytes;
    const float* lse_s = rows_s[stage][0];
    const float* delta_s = rows_s[stage][1];
    // Variant 2: keys of the first block see no query of the second block
    if (kw0 + 31 < split && q0 >= split) continue;
    if (q0 > j0) {
      // interior tile: all four blocks fully visible; blocks software-pipelined
      // MFMA order: sc0 sc1 acc0 sc2 acc1 sc3 acc2 acc3, with the VALU work of block n
      // (P, dS) placed beside the MFMA group that precedes acc(n).
      DkdvBlock b0, b1;
      bf16x8 pfa[2], dsfa[2], pfb[2], dsfb[2];
      dkdv_scores(b0, Qs, dOs, 0, kf, vf, l32, g32);
      __builtin_amdgcn_sched_barrier(0);
      dkdv_scores(b1, Qs, dOs, 1, kf, vf, l32, g32);
      dkdv_softmax<false>(b0, lse_s, delta_s, 0, 0, key, c2, g32, pfa, dsfa);
      interleave_mfma<16, 2, 9>();
      __builtin_amdgcn_sched_barrier(0);
      dkdv_accumulate(dk_acc, dv_acc, Qs, dOs, 0, pfa, dsfa, lane);
      dkdv_softmax<false>(b1, lse_s, delta_s, 1, 0, key, c2, g32, pfb, dsfb);
      interleave_mfma<16, 3, 9>();
      __builtin_amdgcn_sched_barrier(0);
      dkdv_scores(b0, Qs, dOs, 2, kf, vf, l32, g32);
      __builtin_amdgcn_sched_barrier(0);
      dkdv_accumulate(dk_acc, dv_acc, Qs, dOs, 1, pfb, dsfb, lane);
      dkdv_softmax<false>(b0, lse_s, delta_s, 2, 0, key, c2, g32, pfa, dsfa);
      interleave_mfma<16, 3, 9>();
      __builtin_amdgcn_sched_barrier(0);
      dkdv_scores(b1, Qs, dOs, 3, kf, vf, l32, g32);
      __builtin_amdgcn_sched_barrier(0);
      dkdv_accumulate(dk_acc, dv_acc, Qs, dOs, 2, pfa, dsfa, lane);
      dkdv_softmax<false>(b1, lse_s, delta_s, 3, 0, key, c2, g32, pfb, dsfb);
      interleave_mfma<16, 3, 9>();
      __builtin_amdgcn_sched_barrier(0);
      dkdv_accumulate(dk_acc, dv_acc, Qs, dOs, 3, pfb, dsfb, lane);
    } else {
      // diagonal tile: block mb < w is entirely before this wave's keys, block w is masked
      for (int mb = w; mb < 4; ++mb) {
        DkdvBlock blk;
        bf16x8 pf[2], dsf[2];
        dkdv_scores(blk, Qs, dOs, mb, kf, vf, l32, g32);
        if (mb == w) dkdv_softmax<true>(blk, lse_s, delta_s, mb, q0 + 32 * mb, key, c2, g32, pf, dsf);
        else dkdv_softmax<false>(blk, lse_s, delta_s, mb, 0, key, c2, g32, pf, dsf);
        dkdv_accumulate(dk_acc, dv_acc, Qs, dOs, mb, pf, dsf, lane);
      }
    }
  }
  __syncthreads();

  // ---- store dK^T, dV^T blocks (keys lane-indexed) at un-rolled token rows
  if (a.dkv_partial) {
    // kv head shared by both classes: fp32 partial of this class, summed by the combine pass
    const size_t kv_elems = (size_t)a.B * a.N * a.Hkv * 128;
    float* dk_out = a.dkv_partial + (size_t)cls * kv_elems;
    float* dv_out = a.dkv_partial + (size_t)(2 + cls) * kv_elems;
    const int tok = token_of(gidx * a.G + key, s, a.N);
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

// ===========================================================================
// dQ
// ===========================================================================
constexpr int BN = 64;                       // keys per tile
constexpr int kTileBytes = BN * kRowBytes;   // 16 KB

template <bool MASK>
__device__ __forceinline__ void dq_tile(f32x16 (&dq_acc)[4], const bf16x8 (&qf)[8], const bf16x8 (&dof)[8],
                                        const char* Ks, const char* Vs, int j0, int qrow, float c2,
                                        float lse2, float delta, int lane, int l32, int g32) {
  bf16x8 dsf[4];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    f32x16 sa = zero16(), pa = zero16();
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      bf16x8 kr[4], vr[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        kr[i] = frag_rm(Ks, 32 * mb + l32, 2 * (4 * half + i) + g32);
        vr[i] = frag_rm(Vs, 32 * mb + l32, 2 * (4 * half + i) + g32);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        sa = mfma32(kr[i], qf[4 * half + i], sa);
        pa = mfma32(vr[i], dof[4 * half + i], pa);
      }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float e = __builtin_amdgcn_exp2f(fmaf(sa[v], c2, -lse2));
      if (MASK) {
        const int key = j0 + 32 * mb + 8 * (v >> 2) + 4 * g32 + (v & 3);
        if (key > qrow) e = 0.f;
      }
      sa[v] = e * (pa[v] - delta);
    }
    dsf[2 * mb] = pack8(sa[0], sa[1], sa[2], sa[3], sa[4], sa[5], sa[6], sa[7]);
    dsf[2 * mb + 1] = pack8(sa[8], sa[9], sa[10], sa[11], sa[12], sa[13], sa[14], sa[15]);
  }
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    bf16x8 kt[4];
#pragma unroll
    for (int db = 0; db < 4; ++db) kt[db] = frag_tr(Ks, 16 * ks, db, lane);
#pragma unroll
    for (int db = 0; db < 4; ++db) dq_acc[db] = mfma32(kt[db], dsf[ks], dq_acc[db]);
  }
}

__global__ void __launch_bounds__(256, 2)
bwd_dq_bf16_kernel(KArgs a, int T, int n_rest) {
  constexpr int BM = 128;
  __shared__ __attribute__((aligned(1024))) char smem[4 * kTileBytes];   // [stage][K,V]

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
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
  const int qrow = qw0 + l32;
  const int lo_w = qw0 >= split ? split : 0;
  const int jt_first = (i0 >= split ? split : 0) / BN;
  const int jt_diag = i0 / BN;
  const float c2 = a.scale_log2;

  const char* kp = static_cast<const char*>(a.k);
  const char* vp = static_cast<const char*>(a.v);

  bf16x8 qf[8], dof[8];
  float lse2, delta;
  {
    const int tok = token_of(gidx * a.G + qrow, s, a.N);
    const size_t off = ((size_t)((size_t)b * a.N + tok) * a.H + h) * 128;
    const bf16x8* qsrc = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(a.q) + off);
    const bf16x8* dsrc = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(a.dout) + off);
#pragma unroll
    for (int st = 0; st < 8; ++st) { qf[st] = qsrc[2 * st + g32]; dof[st] = dsrc[2 * st + g32]; }
    const size_t ro = ((size_t)b * a.H + h) * a.N + tok;
    lse2 = a.lse[ro] * kLog2e;
    delta = a.delta[ro];
  }

  const uint32_t smem_base = lds_addr(smem);
  const size_t kv_row_bytes = (size_t)a.Hkv * 256;
  const int st_row = 4 * w + (lane >> 4);
  const size_t st_goff = (size_t)st_row * kv_row_bytes + (size_t)(((lane & 15) ^ swz(st_row)) << 4);
  auto issue_tile = [&](int jt, int stage) {
    const int tok0 = token_of(gidx * a.G + jt * BN, s, a.N);
    const size_t base = ((size_t)((size_t)b * a.N + tok0) * a.Hkv + c) * 256 + st_goff;
    const uint32_t ks = smem_base + stage * 2 * kTileBytes + 4 * w * kRowBytes;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      dma16(kp + base + (size_t)p * 16 * kv_row_bytes, ks + 16 * p * kRowBytes);
      dma16(vp + base + (size_t)p * 16 * kv_row_bytes, ks + 16 * p * kRowBytes + kTileBytes);
    }
  };

  f32x16 dq_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) dq_acc[db] = zero16();

  issue_tile(jt_first, 0);
  const int n_tiles = jt_diag + 2 - jt_first;
  for (int n = 0; n < n_tiles; ++n) {
    const int jt = jt_first + n;
    const int stage = n & 1;
    wait_vmcnt0();
    __syncthreads();
    if (n + 1 < n_tiles) issue_tile(jt + 1, stage ^ 1);
    const int j0 = jt * BN;
    const char* Ks = smem + stage * 2 * kTileBytes;
    const char* Vs = Ks + kTileBytes;
    if (j0 + BN - 1 < lo_w) continue;
    if (jt < jt_diag || (jt == jt_diag && w >= 2)) {
      dq_tile<false>(dq_acc, qf, dof, Ks, Vs, j0, qrow, c2, lse2, delta, lane, l32, g32);
    } else if (jt == jt_diag || w >= 2) {
      dq_tile<true>(dq_acc, qf, dof, Ks, Vs, j0, qrow, c2, lse2, delta, lane, l32, g32);
    }
  }
  __syncthreads();

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
