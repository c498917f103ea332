// bf16 S2-Attn forward for gfx950: tiled online-softmax attention inside each group
// of LongLoRA Section 3.2, with the shift of Algorithm 1 folded into row addresses.
//
// One workgroup (4 waves) owns BM = 128*QB consecutive query rows of one
// (batch, head, group) in the head's rolled frame; a wave owns 32*QB of them.  It
// walks the 64-key tiles of the same group up to the diagonal.  Per tile and wave:
//   S^T = K Q^T        A = K rows from LDS (row-major fragments), B = Q^T in registers
//   online softmax     queries are lane-indexed, keys register-indexed, so row max and
//                      row sum are in-lane reductions plus one exchange with lane^32
//   O^T += V^T P^T     A = V^T through transposing LDS reads, B = P^T straight from the
//                      S^T accumulators (no cross-lane movement)
// K/V tiles are staged global -> registers -> LDS with two LDS stages, one barrier per
// tile.  The output tile is transposed through LDS and stored with 16-byte coalesced
// writes at the un-rolled token rows; lse is the natural-log sum of exponentials.
#include "s2attn_bf16_common.h"
#include "s2attn_device.h"
#include "s2attn_launch.h"

namespace s2 {
namespace {

constexpr int BN = 64;                       // keys per tile
constexpr int kTileBytes = BN * kRowBytes;   // 16 KB

template <int QB>
__global__ void __launch_bounds__(256, QB == 1 ? 2 : 1)
fwd_bf16_kernel(KArgs a, int T, int n_rest) {
  constexpr int BM = 128 * QB;
  __shared__ __attribute__((aligned(16))) char smem[4 * kTileBytes];   // [stage][K,V]

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int g32 = lane >> 5, l32 = lane & 31;

  // ---- block -> (batch, head, group, query tile).  Consecutive block ids go to
  // different XCDs, so the id is split as (xcd, slot): every XCD walks its own
  // sequence of (batch, kv head, group) triples, all query heads of the kv head and
  // all query tiles (heaviest first) of a triple back to back, so that the K/V of a
  // group stay in that XCD's L2 while they are being re-read.
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
  const int qw0 = i0 + w * 32 * QB;                 // first query row of this wave
  const int lo_w = qw0 >= split ? split : 0;        // first key visible to this wave
  const int jt_first = (i0 >= split ? split : 0) / BN;
  const int jt_last = (i0 + BM - 1) / BN;
  const float c2 = a.scale_log2;

  const __bf16* qp = static_cast<const __bf16*>(a.q);
  const __bf16* kp = static_cast<const __bf16*>(a.k);
  const __bf16* vp = static_cast<const __bf16*>(a.v);

  // ---- Q^T fragments of this wave, straight from global memory
  bf16x8 qf[QB][8];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int tok = token_of(gidx * a.G + qw0 + 32 * qb + l32, s, a.N);
    const bf16x8* src = reinterpret_cast<const bf16x8*>(qp + ((size_t)((size_t)b * a.N + tok) * a.H + h) * 128);
#pragma unroll
    for (int st = 0; st < 8; ++st) qf[qb][st] = src[2 * st + g32];
  }

  // ---- K/V staging: thread -> (row = tid/16 + 16*pass, 16-byte chunk = tid%16)
  const int ld_row = tid >> 4, ld_chunk = tid & 15;
  uint4 kreg[4], vreg[4];
  auto issue_loads = [&](int jt) {
    const int tok0 = token_of(gidx * a.G + jt * BN, s, a.N);   // a tile never straddles the wrap
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

  f32x16 o_acc[QB][4];
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db) o_acc[qb][db] = zero16();
  }

  issue_loads(jt_first);
  store_lds(0);
  __syncthreads();

  for (int jt = jt_first; jt <= jt_last; ++jt) {
    const int stage = (jt - jt_first) & 1;
    const bool has_next = jt < jt_last;
    if (has_next) issue_loads(jt + 1);
    const int j0 = jt * BN;
    const bool active = (j0 <= qw0 + 32 * QB - 1) && (j0 + BN - 1 >= lo_w);
    if (active) {
      const char* Ks = smem + stage * 2 * kTileBytes;
      const char* Vs = Ks + kTileBytes;
      // S^T tiles: [qb][key block]
      f32x16 s_acc[QB][2];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) { s_acc[qb][0] = zero16(); s_acc[qb][1] = zero16(); }
#pragma unroll
      for (int st = 0; st < 8; ++st) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          const bf16x8 kf = frag_rm(Ks, 32 * mb + l32, 2 * st + g32);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) s_acc[qb][mb] = mfma32(kf, qf[qb][st], s_acc[qb][mb]);
        }
      }
      bf16x8 pf[QB][2][2];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const int qrow0 = qw0 + 32 * qb;
        if (j0 + BN - 1 > qrow0) {   // tile touches the diagonal of this block: causal mask
          const int qrow = qrow0 + l32;
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int key = j0 + 32 * mb + 8 * (v >> 2) + 4 * g32 + (v & 3);
              if (key > qrow) s_acc[qb][mb][v] = -INFINITY;
            }
        }
        float mx = s_acc[qb][0][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s_acc[qb][0][v]);
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s_acc[qb][1][v]);
        mx = max_halves(mx);
        const float m_new = fmaxf(m_run[qb], mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_new) * c2);
        const float mc = m_new * c2;
        float rs = 0.f;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          float p[16];
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            p[v] = __builtin_amdgcn_exp2f(fmaf(s_acc[qb][mb][v], c2, -mc));
            rs += p[v];
          }
          pf[qb][mb][0] = pack8(p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]);
          pf[qb][mb][1] = pack8(p[8], p[9], p[10], p[11], p[12], p[13], p[14], p[15]);
        }
        l_run[qb] = l_run[qb] * alpha + rs;
        m_run[qb] = m_new;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) o_acc[qb][db][v] *= alpha;
      }
      // O^T += V^T P^T
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int db = 0; db < 4; ++db) {
            const bf16x8 vf = frag_tr(Vs, 32 * mb + 16 * t, db, lane);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) o_acc[qb][db] = mfma32(vf, pf[qb][mb][t], o_acc[qb][db]);
          }
    }
    if (has_next) store_lds(stage ^ 1);
    __syncthreads();
  }

  // ---- epilogue: normalise, transpose through LDS, store at un-rolled token rows
  __bf16* op = static_cast<__bf16*>(a.o);
  float l_tot[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    l_tot[qb] = sum_halves(l_run[qb]);
    const float inv = 1.f / l_tot[qb];
    char* Os = smem + (w * QB + qb) * (32 * kRowBytes);
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) {
        const bf16x4 pk = pack4(o_acc[qb][db][4 * vv] * inv, o_acc[qb][db][4 * vv + 1] * inv,
                                o_acc[qb][db][4 * vv + 2] * inv, o_acc[qb][db][4 * vv + 3] * inv);
        *reinterpret_cast<bf16x4*>(Os + tile_off(l32, 4 * db + vv) + 8 * g32) = pk;
      }
  }
  __syncthreads();
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const char* Os = smem + (w * QB + qb) * (32 * kRowBytes);
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = it * 4 + (lane >> 4), ch = lane & 15;
      const uint4 val = *reinterpret_cast<const uint4*>(Os + tile_off(row, ch));
      const int tok = token_of(gidx * a.G + qw0 + 32 * qb + row, s, a.N);
      *reinterpret_cast<uint4*>(op + ((size_t)((size_t)b * a.N + tok) * a.H + h) * 128 + ch * 8) = val;
    }
    if (g32 == 0) {
      const int tok = token_of(gidx * a.G + qw0 + 32 * qb + l32, s, a.N);
      a.lse[((size_t)b * a.H + h) * a.N + tok] = (m_run[qb] * c2 + __builtin_amdgcn_logf(l_tot[qb])) * kLn2;
    }
  }
}

template <int QB>
int launch_fwd_t(const KArgs& a, hipStream_t st) {
  const int T = a.G / (128 * QB);
  const int n_rest = a.B * a.Hkv * (a.N / a.G);
  const int blocks = 8 * T * a.r * ((n_rest + 7) / 8);
  hipLaunchKernelGGL(fwd_bf16_kernel<QB>, dim3(blocks), dim3(256), 0, st, a, T, n_rest);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace

int launch_fwd_bf16(const KArgs& a, hipStream_t st) {
  return launch_fwd_t<1>(a, st);
}

}  // namespace s2
