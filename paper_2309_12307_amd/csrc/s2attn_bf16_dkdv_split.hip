// bf16 S2-Attn backward, dK/dV kernel for gfx950, two waves per SIMD ("role split").
// Used for tile-aligned shapes (G % 128 == 0, shift % 64 == 0, a Variant 2 split that is a
// multiple of 128) with every kv head wholly shifted or unshifted; everything else runs the
// one-wave-per-SIMD kernel of s2attn_bf16_bwd.hip, which computes the same thing.
//
// A workgroup (8 waves on one CU) owns 128 keys of one (batch, kv head, group) in the rolled
// frame of the kv head's class (LongLoRA Algorithm 1: the shift is row addressing only) and
// walks the 64-row query tiles at or below the diagonal (from the end of the group down to
// the diagonal) for every query head of the kv head.  The four products of the
// softmax-Jacobian backward (dS = P * (dP - delta), P recomputed from the stored
// log-sum-exp) are split between the two waves that share a SIMD and a 32-key block, so that
// each fits in 256 registers with all accumulators in ordinary vector registers:
//   wave A (0-3):  S = Q K^T,  P = exp2(c S - lse2)  ->  LDS (fp32),   dV^T += dO^T P
//   wave B (4-7):  delta - dP = delta - dO V^T,  P <- LDS,  dS = P (dP - delta),  dK^T += Q^T dS
// B finishes tile n-1 (dS, dK) at the start of iteration n, after the barrier that also
// publishes the staged tile n, so the hand-over of P costs no barrier of its own, and the
// two waves of a SIMD alternate between the matrix and the vector unit.  Keys are
// lane-indexed and queries register-indexed in S, dP, P and dS, so P and dS are B operands
// as they come out of the accumulators.  Q tiles live in three LDS stages (B still reads
// Q^T of tile n-1 during iteration n), dO tiles, P and the lse / delta rows in two.
// The two query tiles that touch the diagonal run the same code with a causal mask on P;
// blocks wholly above the diagonal are computed with P = 0 rather than branched around.
#include <type_traits>

#include "s2attn_bf16_common.h"
#include "s2attn_device.h"
#include "s2attn_launch.h"

namespace s2 {
namespace {

constexpr int kQT = 64;                            // query rows per tile
constexpr int kQTBytes = kQT * kRowBytes;          // 16 KB
constexpr int kOffQ = 0;                           // 3 stages of Q
constexpr int kOffdO = 3 * kQTBytes;               // 2 stages of dO
constexpr int kOffP = 5 * kQTBytes;                // 2 buffers x 4 key blocks x 2 query blocks x 4 KB (fp32 P)
constexpr int kPBlockBytes = 4096;
constexpr int kPBufBytes = 4 * 2 * kPBlockBytes;   // 32 KB
constexpr int kOffRows = kOffP + 2 * kPBufBytes;   // [2 stages][lse2, delta][64] floats
constexpr int kSmemBytes = kOffRows + 2 * 2 * kQT * 4;

// Scores of both 32-query blocks of a tile against this wave's 32 keys: acc0/acc1 +=
// X[block] Bf^T, X = Q (role A) or dO (role B) read row-major from LDS, Bf = the wave's
// K^T or -V^T fragments.  Steps of 4 MFMAs; every step first issues the reads of the next.
template <int STEP>
__device__ __forceinline__ void sc_load(bf16x8 (&buf)[4], const char* Xs, const LaneOffsets& lo) {
  buf[0] = frag_rm<0>(Xs, lo, 2 * STEP);
  buf[1] = frag_rm<32>(Xs, lo, 2 * STEP);
  buf[2] = frag_rm<0>(Xs, lo, 2 * STEP + 1);
  buf[3] = frag_rm<32>(Xs, lo, 2 * STEP + 1);
}
template <int STEP>
__device__ __forceinline__ void sc_mma(const bf16x8 (&buf)[4], const bf16x8 (&bf)[8], f32x16& acc0, f32x16& acc1) {
  acc0 = mfma32(buf[0], bf[2 * STEP], acc0);
  acc1 = mfma32(buf[1], bf[2 * STEP], acc1);
  acc0 = mfma32(buf[2], bf[2 * STEP + 1], acc0);
  acc1 = mfma32(buf[3], bf[2 * STEP + 1], acc1);
}
__device__ __forceinline__ void scores(f32x16& acc0, f32x16& acc1, const char* Xs, const LaneOffsets& lo,
                                       const bf16x8 (&bf)[8]) {
  bf16x8 fa[4], fb[4], fc[4];
  sc_load<0>(fa, Xs, lo);
  sc_load<1>(fb, Xs, lo);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_setprio(1);   // matrix work goes ahead of the other wave's vector work
  sc_load<2>(fc, Xs, lo); sc_mma<0>(fa, bf, acc0, acc1); __builtin_amdgcn_sched_barrier(0);
  sc_load<3>(fa, Xs, lo); sc_mma<1>(fb, bf, acc0, acc1); __builtin_amdgcn_sched_barrier(0);
  sc_mma<2>(fc, bf, acc0, acc1); __builtin_amdgcn_sched_barrier(0);
  sc_mma<3>(fa, bf, acc0, acc1);
  __builtin_amdgcn_s_setprio(0);
  __builtin_amdgcn_sched_barrier(0);
}

// acc^T (128 x 32 keys) += X^T W for the 64 queries of a tile: X^T = dO^T (role A) or Q^T
// (role B) through transposing LDS reads, W = P or dS as four 16-query B operands.
template <int STEP>
__device__ __forceinline__ void ac_load(bf16x8 (&buf)[4], const char* Xs, const LaneOffsets& lo) {
#pragma unroll
  for (int db = 0; db < 4; ++db) buf[db] = frag_tr<16 * STEP>(Xs, lo, db);
}
__device__ __forceinline__ void ac_mma(const bf16x8 (&buf)[4], bf16x8 wf, f32x16 (&acc)[4]) {
#pragma unroll
  for (int db = 0; db < 4; ++db) acc[db] = mfma32(buf[db], wf, acc[db]);
}
// `fa` and `fb` already hold the fragments of steps 0 and 1 (loaded ahead of the vector work).
__device__ __forceinline__ void accumulate(f32x16 (&acc)[4], bf16x8 (&fa)[4], bf16x8 (&fb)[4], const char* Xs,
                                           const LaneOffsets& lo, const bf16x8 (&wf)[4]) {
  bf16x8 fc[4];
  __builtin_amdgcn_s_setprio(1);
  ac_load<2>(fc, Xs, lo); ac_mma(fa, wf[0], acc); __builtin_amdgcn_sched_barrier(0);
  ac_load<3>(fa, Xs, lo); ac_mma(fb, wf[1], acc); __builtin_amdgcn_sched_barrier(0);
  ac_mma(fc, wf[2], acc); __builtin_amdgcn_sched_barrier(0);
  ac_mma(fa, wf[3], acc);
  __builtin_amdgcn_s_setprio(0);
  __builtin_amdgcn_sched_barrier(0);
}

// 16 bytes per lane, written through to memory (system scope): the stored dS is not read
// again by this kernel, and left to the L2's default policy it evicts the Q and dO tiles that
// the workgroups of an XCD share (measured: 3.6 times the HBM reads).
__device__ __forceinline__ void store_ds(char* dst, bf16x8 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" :: "v"(dst), "v"(v) : "memory");
}

// SPILL: role B also stores dS of every tile it finishes (bf16, the operand it feeds to the
// dK product) for the dQ kernel, which then needs neither S nor dP again.
template <bool SPILL>
__global__ void __launch_bounds__(512, 1)
bwd_dkdv_split_kernel(KArgs a, int T, int il, int n_rest) {
  __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];

  const int tid = threadIdx.x, lane = tid & 63, w = uni(tid >> 6);
  const int g32 = lane >> 5, l32 = lane & 31;
  const bool role_b = w >= 4;
  const int kb = w & 3;

  // block -> (batch, kv head, group, key tile); heaviest key tiles (jt = 0) first
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int y, jt;
  decode_slot(slot, T, il, y, jt);
  int rest = uni(y * 8 + xcd);
  if (rest >= n_rest) return;
  const int NG = uni(a.N / a.G);
  const int gidx = uni(rest % NG); rest = uni(rest / NG);
  const int c = uni(a.c_begin + rest % a.c_count);
  const int b = uni(rest / a.c_count);

  const int h_lo = c * a.r;
  const int s = uni(h_lo >= a.shifted_from ? a.shift : 0);
  const int j0 = jt * 128;
  const int kw0 = j0 + 32 * kb;                      // first key of this wave
  const int key = kw0 + l32;
  // query rows visible to these keys: [j0, G), or [j0, split) for the first block of a split
  // wrap-around group (Variant 2, Appendix B.3; the split is a multiple of the key tile here)
  const int split = uni(split_of_group(a, gidx, s));
  const int nq = uni(((j0 < split ? split : a.G) - j0) / kQT);   // query tiles of one head, >= 2
  const int n_iter = a.r * nq;
  const float c2 = a.scale_log2;

  // loop-invariant B operand of this wave's 32 keys: K^T (role A) or -V^T (role B, so that
  // the accumulator that starts at delta ends as delta - dP)
  bf16x8 bfrag[8];
  {
    const int tok = token_of(gidx * a.G + key, s, a.N);
    const bf16x8* src = reinterpret_cast<const bf16x8*>(
        role_b ? static_cast<const __bf16*>(a.v) + row_off(a.sv, b, tok, c)
               : static_cast<const __bf16*>(a.k) + row_off(a.sk, b, tok, c));
#pragma unroll
    for (int st = 0; st < 8; ++st) bfrag[st] = role_b ? -src[2 * st + g32] : src[2 * st + g32];
  }

  // staging: wave w fills tile rows 4w .. 4w+3 and 32+4w .. 32+4w+3 of Q and of dO; a tile is
  // one contiguous run of 64 tokens: scalar base + fixed per-lane offset
  const uint32_t smem_base = lds_addr(smem);
  const uint64_t q_row_bytes = (uint64_t)a.sq.t * 2, do_row_bytes = (uint64_t)a.so.t * 2;
  const int st_row = 4 * w + (lane >> 4);
  const uint32_t st_chunk = (uint32_t)(((lane & 15) ^ swz(st_row)) << 4);
  const uint32_t q_lane = (uint32_t)(st_row * q_row_bytes) + st_chunk;
  const uint32_t do_lane = (uint32_t)(st_row * do_row_bytes) + st_chunk;
  const uint64_t q_batch = uni64(reinterpret_cast<uint64_t>(a.q) + (uint64_t)b * a.sq.b * 2);
  const uint64_t do_batch = uni64(reinterpret_cast<uint64_t>(a.dout) + (uint64_t)b * a.so.b * 2);
  // tile (hh, it) of the flattened sequence n = hh * nq + it; q_stage = n mod 3, o_stage = n mod 2
  auto issue_tile = [&](int hh, int it, int q_stage, int o_stage) {
    const int h = h_lo + hh;
    const uint32_t tok0 = (uint32_t)token_of(gidx * a.G + j0 + it * kQT, s, a.N);
    const uint64_t qb = uni64(q_batch + tok0 * q_row_bytes + (uint64_t)h * a.sq.h * 2);
    const uint64_t dob = uni64(do_batch + tok0 * do_row_bytes + (uint64_t)h * a.so.h * 2);
    const uint32_t qs = smem_base + kOffQ + q_stage * kQTBytes + 4 * w * kRowBytes;
    const uint32_t dos = smem_base + kOffdO + o_stage * kQTBytes + 4 * w * kRowBytes;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      dma16s(qb + p * 32 * q_row_bytes, q_lane, qs + 32 * p * kRowBytes);
      dma16s(dob + p * 32 * do_row_bytes, do_lane, dos + 32 * p * kRowBytes);
    }
    if (w < 2) {   // wave 0: lse * log2(e), wave 1: delta; 64 rows each
      const uint64_t ro = (((uint64_t)b * a.H + h) * a.N + tok0) * 4;
      const uint32_t dst = smem_base + kOffRows + ((o_stage * 2 + w) * kQT) * 4;
      dma4s(uni64(reinterpret_cast<uint64_t>(w == 0 ? a.lse2 : a.delta) + ro), lane * 4, dst);
    }
  };

  LaneOffsets lo;
  init_lane_offsets(lo, lane);
  f32x16 acc[4];                  // dV^T (role A) or dK^T (role B) of this wave's keys
#pragma unroll
  for (int db = 0; db < 4; ++db) acc[db] = zero16();

  // The flattened tile sequence n = 0 .. r * nq - 1 runs over the query tiles from the end of
  // the group down to the diagonal, all query heads of a tile one after the other.  Every
  // workgroup of a (kv head, group) starts at the last query tile whatever its key tile, so the
  // workgroups that run together read the same Q and dO tile at about the same time and the
  // tile is fetched from HBM once.  (From the diagonal upwards and head by head the
  // workgroups are spread over a window of tiles and, with r heads per kv head, drift apart
  // over r heads' worth of Q and dO: at r = 8 the kernel then reads 8 times as much from HBM
  // and takes 7 % longer; at r = 1 it is 2 % slower.)
  auto advance = [&](int& hh, int& it) {
    if (++hh == a.r) { hh = 0; --it; }
  };
  const int it_first = nq - 1;
  int hh_next = 0, it_next = it_first;     // tile n + 1 (to be staged)
  issue_tile(0, it_first, 0, 0);
  advance(hh_next, it_next);

  if (!role_b) {
    // ------------------------------------------------------------------ role A
    int hh_cur = 0, it = it_first;    // tile n
    int q_st = 0;                     // n mod 3
    for (int n = 0; n <= n_iter; ++n) {
      const int o_st = n & 1;
      wait_vmcnt0();        // this wave's part of tile n has landed
      __syncthreads();      // tile n is complete; everyone has left iteration n-1
      if (n + 1 < n_iter) {
        issue_tile(hh_next, it_next, q_st == 2 ? 0 : q_st + 1, o_st ^ 1);
        advance(hh_next, it_next);
      }
      if (n < n_iter) {
        const char* Qs = smem + kOffQ + q_st * kQTBytes;
        const char* dOs = smem + kOffdO + o_st * kQTBytes;
        const float* lse2_s = reinterpret_cast<const float*>(smem + kOffRows) + (o_st * 2) * kQT;
        char* Px = smem + kOffP + o_st * kPBufBytes + kb * 2 * kPBlockBytes + lane * 16;
        const int q0 = j0 + it * kQT;
        const bool masked = it < 2;   // tiles 0 and 1 touch the diagonal of the 128 keys
        // lse rows of both blocks (queries are register-indexed: 16 values per block and lane
        // half), fetched ahead of the scores so that the vector work below never waits on LDS
        float4 lr[2][4];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int vv = 0; vv < 4; ++vv)
            lr[mb][vv] = *reinterpret_cast<const float4*>(lse2_s + 32 * mb + 8 * vv + 4 * g32);
        f32x16 s0 = zero16(), s1 = zero16();
        scores(s0, s1, Qs, lo, bfrag);
        bf16x8 fa[4], fb[4];
        ac_load<0>(fa, dOs, lo);       // first dO^T fragments arrive during the vector work
        ac_load<1>(fb, dOs, lo);
        bf16x8 pf[4];
        auto softmax_block = [&](auto masked_c, int mb, f32x16& sx) {
          constexpr bool MASKED = decltype(masked_c)::value;
#pragma unroll
          for (int vv = 0; vv < 4; ++vv) {
            const float ls[4] = {lr[mb][vv].x, lr[mb][vv].y, lr[mb][vv].z, lr[mb][vv].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float p = __builtin_amdgcn_exp2f(fmaf(sx[4 * vv + e], c2, -ls[e]));
              if (MASKED && key > q0 + 32 * mb + 8 * vv + 4 * g32 + e) p = 0.f;
              sx[4 * vv + e] = p;
            }
            *reinterpret_cast<float4*>(Px + mb * kPBlockBytes + vv * 1024) =
                make_float4(sx[4 * vv], sx[4 * vv + 1], sx[4 * vv + 2], sx[4 * vv + 3]);
          }
          pf[2 * mb] = pack8(sx[0], sx[1], sx[2], sx[3], sx[4], sx[5], sx[6], sx[7]);
          pf[2 * mb + 1] = pack8(sx[8], sx[9], sx[10], sx[11], sx[12], sx[13], sx[14], sx[15]);
        };
        if (masked) {
          softmax_block(std::true_type{}, 0, s0);
          softmax_block(std::true_type{}, 1, s1);
        } else {
          softmax_block(std::false_type{}, 0, s0);
          softmax_block(std::false_type{}, 1, s1);
        }
        __builtin_amdgcn_sched_barrier(0);
        accumulate(acc, fa, fb, dOs, lo, pf);
      }
      advance(hh_cur, it);
      q_st = q_st == 2 ? 0 : q_st + 1;
    }
  } else {
    // ------------------------------------------------------------------ role B
    int q_st = 0;                     // n mod 3
    f32x16 dp0 = zero16(), dp1 = zero16();   // delta - dP of the pending tile
    // dS blobs of this workgroup: those of key tile jt of head h_lo, one after the other along
    // the query tiles; the next head's are a whole (head, group-count) block further on
    char* ds_lane = nullptr;
    long long ds_head_stride = 0;
    int hh_prev = 0, it_prev = 0;     // tile n - 1 (valid from n = 1 on)
    int hh_cur = 0, it_cur = it_first;   // tile n
    if constexpr (SPILL) {
      const long long per_group = ds_blobs_per_group(T);
      const long long first = ((long long)(b * a.c_count * a.r + (h_lo - a.c_begin * a.r)) * NG + gidx) * per_group +
                              ds_blob_index(T, jt, 0);
      ds_lane = static_cast<char*>(a.ds_spill) + first * kDsBlobBytes + kb * 4096 + lane * 16;
      ds_head_stride = (long long)NG * per_group * kDsBlobBytes;
    }
    for (int n = 0; n <= n_iter; ++n) {
      const int o_st = n & 1;
      wait_vmcnt0();
      __syncthreads();      // also publishes the P of tile n-1
      if (n + 1 < n_iter) {
        issue_tile(hh_next, it_next, q_st == 2 ? 0 : q_st + 1, o_st ^ 1);
        advance(hh_next, it_next);
      }
      const bool has_prev = n >= 1, has_cur = n < n_iter;
      const char* Qs = smem + kOffQ + (q_st == 0 ? 2 : q_st - 1) * kQTBytes;   // tile n-1
      bf16x8 fa[4], fb[4], dsf[4];
      if (has_prev) {
        // finish tile n-1: dS = P * (dP - delta)
        const char* Px = smem + kOffP + (o_st ^ 1) * kPBufBytes + kb * 2 * kPBlockBytes + lane * 16;
        float4 pr[2][4];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int vv = 0; vv < 4; ++vv)
            pr[mb][vv] = *reinterpret_cast<const float4*>(Px + mb * kPBlockBytes + vv * 1024);
        ac_load<0>(fa, Qs, lo);
        ac_load<1>(fb, Qs, lo);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          f32x16& dx = mb == 0 ? dp0 : dp1;
#pragma unroll
          for (int vv = 0; vv < 4; ++vv) {
            const float4 p4 = pr[mb][vv];
            dx[4 * vv + 0] = p4.x * -dx[4 * vv + 0];
            dx[4 * vv + 1] = p4.y * -dx[4 * vv + 1];
            dx[4 * vv + 2] = p4.z * -dx[4 * vv + 2];
            dx[4 * vv + 3] = p4.w * -dx[4 * vv + 3];
          }
          dsf[2 * mb] = pack8(dx[0], dx[1], dx[2], dx[3], dx[4], dx[5], dx[6], dx[7]);
          dsf[2 * mb + 1] = pack8(dx[8], dx[9], dx[10], dx[11], dx[12], dx[13], dx[14], dx[15]);
        }
        if constexpr (SPILL) {
          // the four packed operands as they are: each store is 1 KB of consecutive bytes
          char* dst = ds_lane + hh_prev * ds_head_stride + (long long)it_prev * kDsBlobBytes;
#pragma unroll
          for (int f = 0; f < 4; ++f)
            store_ds(dst + 1024 * f, dsf[f]);
        }
      }
      if constexpr (SPILL) {   // tile n becomes tile n - 1
        hh_prev = hh_cur; it_prev = it_cur;
        advance(hh_cur, it_cur);
      }
      if (has_cur) {
        // delta - dP of tile n: the accumulators start at delta (per query row = per register);
        // the rows are fetched here so that they arrive during the matrix work below
        const float* delta_s = reinterpret_cast<const float*>(smem + kOffRows) + (o_st * 2 + 1) * kQT;
#pragma unroll
        for (int vv = 0; vv < 4; ++vv) {
          const float4 d0 = *reinterpret_cast<const float4*>(delta_s + 8 * vv + 4 * g32);
          const float4 d1 = *reinterpret_cast<const float4*>(delta_s + 32 + 8 * vv + 4 * g32);
          dp0[4 * vv] = d0.x; dp0[4 * vv + 1] = d0.y; dp0[4 * vv + 2] = d0.z; dp0[4 * vv + 3] = d0.w;
          dp1[4 * vv] = d1.x; dp1[4 * vv + 1] = d1.y; dp1[4 * vv + 2] = d1.z; dp1[4 * vv + 3] = d1.w;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (has_prev) accumulate(acc, fa, fb, Qs, lo, dsf);   // dK^T += Q^T dS
      if (has_cur) scores(dp0, dp1, smem + kOffdO + o_st * kQTBytes, lo, bfrag);
      q_st = q_st == 2 ? 0 : q_st + 1;
    }
  }
  __syncthreads();

  // ---- store this wave's 32 x 128 block (dV for role A, dK for role B) at un-rolled rows
  char* region = smem + w * (32 * kRowBytes);
  acc_to_lds(region, acc, role_b ? a.scale : 1.f, l32, g32);
  __syncthreads();
  __bf16* outp = static_cast<__bf16*>(role_b ? a.dk : a.dv);
  const TStride so = role_b ? a.sdk : a.sdv;
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int row = it * 4 + (lane >> 4), ch = lane & 15;
    const int tok = token_of(gidx * a.G + kw0 + row, s, a.N);
    *reinterpret_cast<uint4*>(outp + row_off(so, b, tok, c) + ch * 8) =
        *reinterpret_cast<const uint4*>(region + tile_off(row, ch));
  }
}

}  // namespace

bool dkdv_split_applies(const KArgs& a) {
  return !a.ragged && !a.mixed;
}

int launch_bwd_dkdv_split_bf16(const KArgs& a, hipStream_t st) {
  const int NG = a.N / a.G;
  const int T = a.G / 128;
  const int n_rest = a.B * a.c_count * NG;
  const int il = interleave_for(T, 32);   // 32 CUs per XCD, one workgroup each
  const int blocks = 8 * T * pad_to((n_rest + 7) / 8, il);
  if (a.ds_spill)
    hipLaunchKernelGGL(bwd_dkdv_split_kernel<true>, dim3(blocks), dim3(512), 0, st, a, T, il, n_rest);
  else
    hipLaunchKernelGGL(bwd_dkdv_split_kernel<false>, dim3(blocks), dim3(512), 0, st, a, T, il, n_rest);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace s2
