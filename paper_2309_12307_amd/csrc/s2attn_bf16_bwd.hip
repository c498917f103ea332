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
#include <type_traits>

#include "s2attn_bf16_common.h"
#include "s2attn_device.h"
#include "s2attn_launch.h"

namespace s2 {
namespace {

// ===========================================================================
// dK / dV
// ===========================================================================
constexpr int kQTileRows = 128;
constexpr int kQTileBytes = kQTileRows * kRowBytes;   // 32 KB

struct DkdvBlock {     // S and dP accumulators of one 32-query block
  f32x16 s, dp;
};

struct DkdvTile {      // the staged query tile and per-lane constants
  const char* Qs;
  const char* dOs;
  const float* lse2_s;
  const float* delta_s;
  float c2;
  int g32;
  LaneOffsets lo;
};

// ---- fragment loads and MFMA groups, one "phase" = 8 MFMAs fed by 8 fragments
// scores phase (block MB, k-steps 4H..4H+3): S += Q K^T, dP += dO V^T
template <int MB, int H>
__device__ __forceinline__ void load_sc(bf16x8 (&buf)[8], const DkdvTile& t) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    buf[i] = frag_rm<32 * MB>(t.Qs, t.lo, 4 * H + i);
    buf[4 + i] = frag_rm<32 * MB>(t.dOs, t.lo, 4 * H + i);
  }
}
template <int H>
__device__ __forceinline__ void mma_sc(const bf16x8 (&buf)[8], DkdvBlock& blk, const bf16x8 (&kf)[8],
                                       const bf16x8 (&vf)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    blk.s = mfma32(buf[i], kf[4 * H + i], blk.s);
    blk.dp = mfma32(buf[4 + i], vf[4 * H + i], blk.dp);
  }
}
// accumulate phase (block MB, queries 16T..16T+15 of it): dV^T += dO^T P, dK^T += Q^T dS.
// DH: head dimension the products run over (128, or 64 when the upper half of every tile row is
// zero padding).
template <int MB, int T, int DH = 128>
__device__ __forceinline__ void load_acc(bf16x8 (&buf)[8], const DkdvTile& t) {
#pragma unroll
  for (int db = 0; db < DH / 32; ++db) {
    buf[db] = frag_tr<32 * MB + 16 * T>(t.dOs, t.lo, db);
    buf[4 + db] = frag_tr<32 * MB + 16 * T>(t.Qs, t.lo, db);
  }
}
template <int T, int DH = 128>
__device__ __forceinline__ void mma_acc(const bf16x8 (&buf)[8], const bf16x4 (&pq)[4], const bf16x4 (&dsq)[4],
                                        f32x16 (&dk_acc)[4], f32x16 (&dv_acc)[4]) {
  const bf16x8 pf = __builtin_shufflevector(pq[2 * T], pq[2 * T + 1], 0, 1, 2, 3, 4, 5, 6, 7);
  const bf16x8 dsf = __builtin_shufflevector(dsq[2 * T], dsq[2 * T + 1], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
  for (int db = 0; db < DH / 32; ++db) {
    dv_acc[db] = mfma32(buf[db], pf, dv_acc[db]);
    dk_acc[db] = mfma32(buf[4 + db], dsf, dk_acc[db]);
  }
}
// The dP accumulator of block MB starts at delta (per query row, i.e. per register) and the
// V fragments are negated, so that the accumulator ends as delta - dP and dS = P * -(that)
// needs no subtraction.
template <int MB>
__device__ __forceinline__ void init_dp(DkdvBlock& blk, const DkdvTile& t) {
#pragma unroll
  for (int qtr = 0; qtr < 4; ++qtr) {
    const float4 d4 = *reinterpret_cast<const float4*>(t.delta_s + 32 * MB + 8 * qtr + 4 * t.g32);
    blk.dp[4 * qtr] = d4.x; blk.dp[4 * qtr + 1] = d4.y; blk.dp[4 * qtr + 2] = d4.z; blk.dp[4 * qtr + 3] = d4.w;
  }
}

// P and dS for accumulator registers 4*QTR .. 4*QTR+3 of block MB (4 consecutive queries
// per lane half), packed to bf16.  MASK: causal mask against this lane's key, and query
// rows at or past q_lim (padding of a partial tile) contribute nothing.
template <int MB, int QTR, bool MASK>
__device__ __forceinline__ void sm_quarter(const DkdvBlock& blk, const DkdvTile& t, bf16x4& pq, bf16x4& dsq,
                                           int q_first = 0, int key = 0, int q_lim = INT32_MAX) {
  const float4 l4 = *reinterpret_cast<const float4*>(t.lse2_s + 32 * MB + 8 * QTR + 4 * t.g32);
  const float ls[4] = {l4.x, l4.y, l4.z, l4.w};
  float p[4], ds[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int v = 4 * QTR + e;
    float pv = __builtin_amdgcn_exp2f(fmaf(blk.s[v], t.c2, -ls[e]));
    if (MASK) {
      const int qrow = q_first + 8 * QTR + 4 * t.g32 + e;
      if (key > qrow || qrow >= q_lim) pv = 0.f;
    }
    p[e] = pv;
    ds[e] = pv * -blk.dp[v];
  }
  pq = pack4(p[0], p[1], p[2], p[3]);
  dsq = pack4(ds[0], ds[1], ds[2], ds[3]);
}

// Interior tile (all 4 x 32 queries visible to all 32 keys of the wave): 16 phases of
// 8 MFMAs.  MFMA order per block n: scores(n), then accumulate(n) one block later, so
// that the VALU work of block n (four quarters) always has independent MFMAs of blocks
// n-1 / n+1 beside it; every phase also issues the LDS reads of the next phase into the
// other fragment buffer.
__device__ __forceinline__ void dkdv_interior_tile(const DkdvTile& t, const bf16x8 (&kf)[8], const bf16x8 (&vf)[8],
                                                   f32x16 (&dk_acc)[4], f32x16 (&dv_acc)[4]) {
#define S2_PHASE_END(DS, VA) interleave_mfma2<3, 6, 5, 2 * VA>(); __builtin_amdgcn_sched_barrier(0)
  bf16x8 fa[8], fb[8];
  DkdvBlock b0, b1;
  bf16x4 pa[4], da[4], pb[4], db[4];
  load_sc<0, 0>(fa, t);
  __builtin_amdgcn_sched_barrier(0);
  // 1-2: scores(0)
  load_sc<0, 1>(fb, t); b0.s = zero16(); init_dp<0>(b0, t); mma_sc<0>(fa, b0, kf, vf); S2_PHASE_END(1, 0);
  load_sc<1, 0>(fa, t); mma_sc<1>(fb, b0, kf, vf); S2_PHASE_END(1, 0);
  // 3-4: scores(1) | softmax(0)
  load_sc<1, 1>(fb, t); b1.s = zero16(); init_dp<1>(b1, t); mma_sc<0>(fa, b1, kf, vf);
  sm_quarter<0, 0, false>(b0, t, pa[0], da[0]); sm_quarter<0, 1, false>(b0, t, pa[1], da[1]); S2_PHASE_END(2, 8);
  load_acc<0, 0>(fa, t); mma_sc<1>(fb, b1, kf, vf);
  sm_quarter<0, 2, false>(b0, t, pa[2], da[2]); sm_quarter<0, 3, false>(b0, t, pa[3], da[3]); S2_PHASE_END(3, 8);
  // 5-6: accumulate(0) | softmax(1) first half
  load_acc<0, 1>(fb, t); mma_acc<0>(fa, pa, da, dk_acc, dv_acc); sm_quarter<1, 0, false>(b1, t, pb[0], db[0]); S2_PHASE_END(3, 4);
  load_sc<2, 0>(fa, t); mma_acc<1>(fb, pa, da, dk_acc, dv_acc); sm_quarter<1, 1, false>(b1, t, pb[1], db[1]); S2_PHASE_END(2, 4);
  // 7-8: scores(2) | softmax(1) second half
  load_sc<2, 1>(fb, t); b0.s = zero16(); init_dp<2>(b0, t); mma_sc<0>(fa, b0, kf, vf);
  sm_quarter<1, 2, false>(b1, t, pb[2], db[2]); S2_PHASE_END(2, 4);
  load_acc<1, 0>(fa, t); mma_sc<1>(fb, b0, kf, vf); sm_quarter<1, 3, false>(b1, t, pb[3], db[3]); S2_PHASE_END(3, 4);
  // 9-10: accumulate(1) | softmax(2) first half
  load_acc<1, 1>(fb, t); mma_acc<0>(fa, pb, db, dk_acc, dv_acc); sm_quarter<2, 0, false>(b0, t, pa[0], da[0]); S2_PHASE_END(3, 4);
  load_sc<3, 0>(fa, t); mma_acc<1>(fb, pb, db, dk_acc, dv_acc); sm_quarter<2, 1, false>(b0, t, pa[1], da[1]); S2_PHASE_END(2, 4);
  // 11-12: scores(3) | softmax(2) second half
  load_sc<3, 1>(fb, t); b1.s = zero16(); init_dp<3>(b1, t); mma_sc<0>(fa, b1, kf, vf);
  sm_quarter<2, 2, false>(b0, t, pa[2], da[2]); S2_PHASE_END(2, 4);
  load_acc<2, 0>(fa, t); mma_sc<1>(fb, b1, kf, vf); sm_quarter<2, 3, false>(b0, t, pa[3], da[3]); S2_PHASE_END(3, 4);
  // 13-14: accumulate(2) | softmax(3) first half
  load_acc<2, 1>(fb, t); mma_acc<0>(fa, pa, da, dk_acc, dv_acc); sm_quarter<3, 0, false>(b1, t, pb[0], db[0]); S2_PHASE_END(3, 4);
  load_acc<3, 0>(fa, t); mma_acc<1>(fb, pa, da, dk_acc, dv_acc); sm_quarter<3, 1, false>(b1, t, pb[1], db[1]); S2_PHASE_END(3, 4);
  // 15-16: accumulate(3) | softmax(3) second half
  load_acc<3, 1>(fb, t); mma_acc<0>(fa, pb, db, dk_acc, dv_acc);
  sm_quarter<3, 2, false>(b1, t, pb[2], db[2]); sm_quarter<3, 3, false>(b1, t, pb[3], db[3]); S2_PHASE_END(3, 8);
  mma_acc<1>(fb, pb, db, dk_acc, dv_acc);
  __builtin_amdgcn_sched_barrier(0);
#undef S2_PHASE_END
}

// One 32-query block without pipelining (diagonal tiles; every tile when the head dimension is 64).
template <bool MASK, int DH = 128>
__device__ __forceinline__ void dkdv_block(const DkdvTile& t, int mb, int q_first, int key, const bf16x8 (&kf)[8],
                                           const bf16x8 (&vf)[8], f32x16 (&dk_acc)[4], f32x16 (&dv_acc)[4],
                                           int q_lim = INT32_MAX) {
  DkdvTile tt = t;
  tt.Qs += mb * 32 * kRowBytes;     // rows of a tile are swizzled by (row & 15) only, so a
  tt.dOs += mb * 32 * kRowBytes;    // block is addressed by moving the base by 32 rows
  tt.lse2_s += 32 * mb;
  tt.delta_s += 32 * mb;
  bf16x8 fa[8], fb[8];
  DkdvBlock blk;
  bf16x4 pq[4], dsq[4];
  blk.s = zero16(); init_dp<0>(blk, tt);
  load_sc<0, 0>(fa, tt);
  if constexpr (DH == 128) load_sc<0, 1>(fb, tt);
  mma_sc<0>(fa, blk, kf, vf);
  if constexpr (DH == 128) mma_sc<1>(fb, blk, kf, vf);
  load_acc<0, 0, DH>(fa, tt); load_acc<0, 1, DH>(fb, tt);
  sm_quarter<0, 0, MASK>(blk, tt, pq[0], dsq[0], q_first, key, q_lim);
  sm_quarter<0, 1, MASK>(blk, tt, pq[1], dsq[1], q_first, key, q_lim);
  sm_quarter<0, 2, MASK>(blk, tt, pq[2], dsq[2], q_first, key, q_lim);
  sm_quarter<0, 3, MASK>(blk, tt, pq[3], dsq[3], q_first, key, q_lim);
  mma_acc<0, DH>(fa, pq, dsq, dk_acc, dv_acc);
  mma_acc<1, DH>(fb, pq, dsq, dk_acc, dv_acc);
}

// RAGGED: G is not a multiple of 128 or the shift not of 64 -- tiles may be partial and
// the wrap point may fall inside one, so every staged row finds its own token and the
// padding rows of the last tile are masked.  The aligned instantiation carries none of it.
// DH = 64 (only with RAGGED): the head dimension is 64 and the products skip the zero half.
template <bool RAGGED, int DH = 128>
__global__ void __launch_bounds__(256, 1)
bwd_dkdv_bf16_kernel(KArgs a, int ncls, int T, int il, int n_rest) {
  __shared__ __attribute__((aligned(1024))) char smem[4 * kQTileBytes];            // [stage][Q,dO]
  __shared__ __attribute__((aligned(1024))) float rows_s[2][2][kQTileRows];        // [stage][lse * log2(e), delta]

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g32 = lane >> 5, l32 = lane & 31;

  // block -> (batch, kv head, class, group, key tile); heaviest key tiles (jt = 0) first
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int y, jt;
  decode_slot(slot, T, il, y, jt);
  int rest = uni(y * 8 + xcd);
  if (rest >= n_rest) return;
  const int NG = uni(a.N / a.G);
  const int gidx = uni(rest % NG); rest = uni(rest / NG);
  const int cls_slot = uni(rest % ncls); rest = uni(rest / ncls);
  const int c = uni(rest % a.Hkv);
  const int b = uni(rest / a.Hkv);

  int h_lo = c * a.r, h_hi = (c + 1) * a.r;
  const int cls = ncls == 2 ? cls_slot : (h_lo >= a.shifted_from ? 1 : 0);
  if (cls == 0) h_hi = min(h_hi, a.shifted_from); else h_lo = max(h_lo, a.shifted_from);
  const int nheads = uni(max(h_hi - h_lo, 0));
  h_lo = uni(h_lo);

  const int s = uni(cls ? a.shift : 0);
  // the causal run this block works in (see the forward kernel): the aligned kernel cuts the
  // query range of a split wrap-around group at `split`, a multiple of the tile; the ragged
  // one runs the two blocks as runs of their own
  Run run{gidx * a.G, a.G};
  int split = uni(split_of_group(a, gidx, s));
  if constexpr (RAGGED) {
    if (!run_of_tile(a, gidx, s, kQTileRows, jt, run)) return;
    run.p0 = uni(run.p0); run.len = uni(run.len);
    split = run.len;
  }
  const int j0 = jt * 128;
  const int kw0 = j0 + 32 * w;                       // first key of this wave
  const int key = kw0 + l32;
  // query rows visible to this workgroup's keys: [j0, q_end)
  const int q_end = uni((j0 < split) ? split : run.len);
  const int it_begin = uni(j0 / kQTileRows);
  const int nq = uni((q_end - j0 + kQTileRows - 1) / kQTileRows);
  const int n_iter = nheads * nq;
  const float c2 = a.scale_log2;

  const char* qp = static_cast<const char*>(a.q);
  const char* dop = static_cast<const char*>(a.dout);

  // K^T and -V^T fragments of this wave's 32 keys (the sign: see init_dp)
  bf16x8 kf[8], vf[8];
  {
    const int tok = run_token(a, run, key, s);
    const bf16x8* ksrc = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(a.k) + row_off(a.sk, b, tok, c));
    const bf16x8* vsrc = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(a.v) + row_off(a.sv, b, tok, c));
#pragma unroll
    for (int st = 0; st < DH / 16; ++st) { kf[st] = ksrc[2 * st + g32]; vf[st] = -vsrc[2 * st + g32]; }
  }

  // staging: wave w, pass p fills tile rows 16p + 4w .. +3 (1 KB); in the aligned case
  // (shift and G multiples of 64) every 64 rows of a tile are one contiguous token run.
  const uint32_t smem_base = lds_addr(smem);
  const uint32_t rows_base = lds_addr(rows_s);
  const uint64_t q_row_bytes = (uint64_t)a.sq.t * 2, do_row_bytes = (uint64_t)a.so.t * 2;
  const int st_row = 4 * w + (lane >> 4);
  const uint32_t st_chunk = (uint32_t)(((lane & 15) ^ swz(st_row)) << 4);
  // aligned staging: scalar base of a 64-row token run plus these per-lane offsets
  const uint32_t q_lane = (uint32_t)(st_row * q_row_bytes) + st_chunk;
  const uint32_t do_lane = (uint32_t)(st_row * do_row_bytes) + st_chunk;
  const uint64_t q_batch = uni64(reinterpret_cast<uint64_t>(qp) + (uint64_t)b * a.sq.b * 2);
  const uint64_t do_batch = uni64(reinterpret_cast<uint64_t>(dop) + (uint64_t)b * a.so.b * 2);
  auto issue_tile = [&](int hh, int it, int stage) __attribute__((always_inline)) {
    const int h = h_lo + hh;
    const int q0 = (it_begin + it) * kQTileRows;
    const uint32_t qs = smem_base + stage * 2 * kQTileBytes + 4 * w * kRowBytes;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      if constexpr (!RAGGED) {
        const uint32_t tok0 = (uint32_t)token_of(run.p0 + q0 + 64 * hf, s, a.N);
        const uint64_t qb = q_batch + tok0 * q_row_bytes + (uint64_t)h * a.sq.h * 2;
        const uint64_t dob = do_batch + tok0 * do_row_bytes + (uint64_t)h * a.so.h * 2;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          dma16s(qb + p * 16 * q_row_bytes, q_lane, qs + (64 * hf + 16 * p) * kRowBytes);
          dma16s(dob + p * 16 * do_row_bytes, do_lane, qs + (64 * hf + 16 * p) * kRowBytes + kQTileBytes);
        }
        if (w == hf) {   // wave 0 / 1: lse and delta of rows 64*hf .. +63
          const uint64_t ro = (((uint64_t)b * a.H + h) * a.N + tok0) * 4;
          dma4s(reinterpret_cast<uint64_t>(a.lse2) + ro, lane * 4, rows_base + ((stage * 2 + 0) * kQTileRows + 64 * hf) * 4);
          dma4s(reinterpret_cast<uint64_t>(a.delta) + ro, lane * 4, rows_base + ((stage * 2 + 1) * kQTileRows + 64 * hf) * 4);
        }
      } else {   // every row finds its own token; padding rows repeat the last row of the run
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int tok = run_token(a, run, q0 + 64 * hf + 16 * p + st_row, s);
          if (DH == 64 && st_chunk >= 2 * DH) continue;   // a 64-wide row fills the first eight chunks only
          dma16(qp + row_off(a.sq, b, tok, h) * 2 + st_chunk, qs + (64 * hf + 16 * p) * kRowBytes);
          dma16(dop + row_off(a.so, b, tok, h) * 2 + st_chunk,
                qs + (64 * hf + 16 * p) * kRowBytes + kQTileBytes);
        }
        if (w == hf) {
          const size_t ro = ((size_t)b * a.H + h) * a.N + run_token(a, run, q0 + 64 * hf + lane, s);
          dma4(a.lse2 + ro, rows_base + ((stage * 2 + 0) * kQTileRows + 64 * hf) * 4);
          dma4(a.delta + ro, rows_base + ((stage * 2 + 1) * kQTileRows + 64 * hf) * 4);
        }
      }
    }
  };

  LaneOffsets lo;
  init_lane_offsets(lo, lane);
  f32x16 dk_acc[4], dv_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) { dk_acc[db] = zero16(); dv_acc[db] = zero16(); }

  // The n-th tile of the walk is query tile it_begin + it of head h_lo + hh.  Waits for its
  // staged data, starts the staging of the next one (the next head of the same query tile,
  // else the first head of the tile before) into the other stage and describes the tile.
  auto begin_tile = [&](int n, int hh, int it) __attribute__((always_inline)) {
    const int stage = n & 1;
    wait_vmcnt0();
    __syncthreads();
    if (n + 1 < n_iter) {
      const bool wrap = hh + 1 == nheads;
      issue_tile(wrap ? 0 : hh + 1, wrap ? it - 1 : it, stage ^ 1);
    }
    if constexpr (RAGGED) __builtin_amdgcn_sched_barrier(0);   // keeps the per-row addresses out of the tile body
    DkdvTile t;
    t.Qs = smem + stage * 2 * kQTileBytes;
    t.dOs = t.Qs + kQTileBytes;
    t.lse2_s = rows_s[stage][0];
    t.delta_s = rows_s[stage][1];
    t.c2 = c2; t.g32 = g32; t.lo = lo;
    return t;
  };

  // Query tiles from the end of the run down to the diagonal, the heads of the kv head
  // innermost: workgroups of one (group, class) that hold different key tiles then ask for
  // the same Q / dO tile at about the same time, whatever their number of tiles, and the L2
  // serves all but the first.  The partial last tile (a group size that is not a multiple of
  // the tile) comes first, the interior tiles follow in a loop of their own (the hot loop
  // holds nothing but the pipelined interior tile), the diagonal tiles come last.
  const bool has_tail = RAGGED && (run.len % kQTileRows != 0);
  const int n_full = has_tail ? nq - 1 : nq;           // tiles [0, n_full) are complete
  if (n_iter > 0) issue_tile(0, nq - 1, 0);
  int n = 0;
  if (has_tail && nq > 1) {
    const int q0 = j0 + (nq - 1) * kQTileRows;
    for (int hh = 0; hh < nheads; ++hh, ++n) {
      const DkdvTile t = begin_tile(n, hh, nq - 1);
      for (int mb = 0; mb < 4; ++mb) dkdv_block<true, DH>(t, mb, q0 + 32 * mb, key, kf, vf, dk_acc, dv_acc, run.len);
    }
  }
  for (int it = n_full - 1; it >= 1; --it) {
    for (int hh = 0; hh < nheads; ++hh, ++n) {
      const DkdvTile t = begin_tile(n, hh, it);
      if constexpr (DH == 128) {
        dkdv_interior_tile(t, kf, vf, dk_acc, dv_acc);
      } else {
        for (int mb = 0; mb < 4; ++mb) dkdv_block<false, DH>(t, mb, 0, key, kf, vf, dk_acc, dv_acc);
      }
    }
  }
  for (int hh = 0; hh < nheads; ++hh, ++n) {
    const DkdvTile t = begin_tile(n, hh, 0);
    if constexpr (RAGGED) {
      // query rows >= G (padding of a partial tile) give P = 0; blocks before this wave's
      // keys are skipped
      for (int mb = w; mb < 4; ++mb) dkdv_block<true, DH>(t, mb, j0 + 32 * mb, key, kf, vf, dk_acc, dv_acc, run.len);
    } else {
      // block mb < w is entirely before this wave's keys, block w is masked
      dkdv_block<true>(t, w, j0 + 32 * w, key, kf, vf, dk_acc, dv_acc);
      for (int mb = w + 1; mb < 4; ++mb) dkdv_block<false>(t, mb, 0, key, kf, vf, dk_acc, dv_acc);
    }
  }
  __syncthreads();

  // ---- store dK^T, dV^T blocks (keys lane-indexed) at un-rolled token rows
  if (a.dkv_partial) {
    // kv head shared by both classes: fp32 partial of this class, summed by the combine pass
    const size_t kv_elems = (size_t)a.B * a.N * a.Hkv * a.D;
    float* dk_out = a.dkv_partial + (size_t)cls * kv_elems;
    float* dv_out = a.dkv_partial + (size_t)(2 + cls) * kv_elems;
    if (key >= run.len) return;   // padding key of a partial tile
    const int tok = token_of(run.p0 + key, s, a.N);
    const size_t base = ((size_t)((size_t)b * a.N + tok) * a.Hkv + c) * a.D;   // partials are contiguous
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) {
        const int d = 32 * db + 8 * vv + 4 * g32;
        if (d >= a.D) continue;   // head dimension 64: the upper half of the tile is padding
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
    if (kw0 + row >= run.len || ch * 8 >= a.D) continue;   // padding key of a partial tile, padding of a narrow row
    const int tok = token_of(run.p0 + kw0 + row, s, a.N);
    *reinterpret_cast<uint4*>(dkp + row_off(a.sdk, b, tok, c) + ch * 8) =
        *reinterpret_cast<const uint4*>(rk + tile_off(row, ch));
    *reinterpret_cast<uint4*>(dvp + row_off(a.sdv, b, tok, c) + ch * 8) =
        *reinterpret_cast<const uint4*>(rv + tile_off(row, ch));
  }
}

// ===========================================================================
// dQ
// ===========================================================================
constexpr int BN = 64;                       // keys per tile
constexpr int kTileBytes = BN * kRowBytes;   // 16 KB

// One 64-key tile of the dQ kernel as 12 steps of 4 MFMAs, each fed by 4 fragments:
//   steps 0-3 / 4-7: S^T and dP^T of key block 0 / 1 over d = 32j .. 32j+31
//   steps 8-11:      dQ^T += K^T dS^T for keys 16k .. 16k+15
// Every step first issues the LDS reads of the next step into the other fragment buffer
// (also across the exp/multiply sections), then runs its own four MFMAs.
template <int STEP>
__device__ __forceinline__ void dq_load(bf16x8 (&buf)[4], const char* Ks, const char* Vs, const LaneOffsets& lo) {
  if constexpr (STEP < 8) {
    constexpr int ROW0 = 32 * (STEP / 4), J = STEP % 4;
    buf[0] = frag_rm<ROW0>(Ks, lo, 2 * J);
    buf[1] = frag_rm<ROW0>(Vs, lo, 2 * J);
    buf[2] = frag_rm<ROW0>(Ks, lo, 2 * J + 1);
    buf[3] = frag_rm<ROW0>(Vs, lo, 2 * J + 1);
  } else {
#pragma unroll
    for (int db = 0; db < 4; ++db) buf[db] = frag_tr<16 * (STEP - 8)>(Ks, lo, db);
  }
}

template <int STEP>
__device__ __forceinline__ void dq_mma(const bf16x8 (&buf)[4], const bf16x8 (&qf)[8], const bf16x8 (&dof)[8],
                                       f32x16& sa, f32x16& pa, const bf16x8 (&dsf)[4], f32x16 (&dq_acc)[4]) {
  if constexpr (STEP < 8) {
    constexpr int J = STEP % 4;
    sa = mfma32(buf[0], qf[2 * J], sa);
    pa = mfma32(buf[1], dof[2 * J], pa);
    sa = mfma32(buf[2], qf[2 * J + 1], sa);
    pa = mfma32(buf[3], dof[2 * J + 1], pa);
  } else {
#pragma unroll
    for (int db = 0; db < 4; ++db) dq_acc[db] = mfma32(buf[db], dsf[STEP - 8], dq_acc[db]);
  }
}

// dS^T = P^T * (dP^T - delta) of one 32-key block, packed as two B operands.
template <int ROW0>
__device__ __forceinline__ void dq_ds(f32x16& sa, const f32x16& pa, bf16x8& ds_lo, bf16x8& ds_hi, int j0, int qrow,
                                      float c2, float lse2, float delta, int g32, bool masked) {
  if (masked) {   // wave-uniform: exp2(-inf) = 0 removes keys after the query
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = j0 + ROW0 + 8 * (v >> 2) + 4 * g32 + (v & 3);
      if (key > qrow) sa[v] = -INFINITY;
    }
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) sa[v] = __builtin_amdgcn_exp2f(fmaf(sa[v], c2, -lse2)) * (pa[v] - delta);
  ds_lo = pack8(sa[0], sa[1], sa[2], sa[3], sa[4], sa[5], sa[6], sa[7]);
  ds_hi = pack8(sa[8], sa[9], sa[10], sa[11], sa[12], sa[13], sa[14], sa[15]);
}

__device__ __forceinline__ void dq_tile(f32x16 (&dq_acc)[4], const bf16x8 (&qf)[8], const bf16x8 (&dof)[8],
                                        const char* Ks, const char* Vs, const LaneOffsets& lo, int j0,
                                        int qrow, float c2, float lse2, float delta, int g32, bool masked) {
#define S2_DQ_STEP(N, CUR, NXT)                                   \
  dq_load<N + 1>(NXT, Ks, Vs, lo);                                \
  dq_mma<N>(CUR, qf, dof, sa, pa, dsf, dq_acc);                   \
  __builtin_amdgcn_sched_barrier(0)
  bf16x8 fa[4], fb[4], dsf[4];
  f32x16 sa = zero16(), pa = zero16();
  dq_load<0>(fa, Ks, Vs, lo);
  __builtin_amdgcn_sched_barrier(0);
  S2_DQ_STEP(0, fa, fb);
  S2_DQ_STEP(1, fb, fa);
  S2_DQ_STEP(2, fa, fb);
  S2_DQ_STEP(3, fb, fa);            // loads step 4 (block 1) before the vector section
  dq_ds<0>(sa, pa, dsf[0], dsf[1], j0, qrow, c2, lse2, delta, g32, masked);
  sa = zero16();
  pa = zero16();
  __builtin_amdgcn_sched_barrier(0);
  S2_DQ_STEP(4, fa, fb);
  S2_DQ_STEP(5, fb, fa);
  S2_DQ_STEP(6, fa, fb);
  S2_DQ_STEP(7, fb, fa);            // loads step 8 (first K^T fragments)
  dq_ds<32>(sa, pa, dsf[2], dsf[3], j0, qrow, c2, lse2, delta, g32, masked);
  __builtin_amdgcn_sched_barrier(0);
  S2_DQ_STEP(8, fa, fb);
  S2_DQ_STEP(9, fb, fa);
  S2_DQ_STEP(10, fa, fb);
  dq_mma<11>(fb, qf, dof, sa, pa, dsf, dq_acc);
#undef S2_DQ_STEP
}

// Head dimension 64 (the upper half of every tile row is zero padding): the same three
// products over d = 0 .. 63 only, one 32-key block after the other, without the step pipeline.
template <int ROW0>
__device__ __forceinline__ void dq_scores64(f32x16& sa, f32x16& pa, const bf16x8 (&qf)[8], const bf16x8 (&dof)[8],
                                            const char* Ks, const char* Vs, const LaneOffsets& lo) {
  bf16x8 kfr[4], vfr[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) { kfr[k] = frag_rm<ROW0>(Ks, lo, k); vfr[k] = frag_rm<ROW0>(Vs, lo, k); }
#pragma unroll
  for (int k = 0; k < 4; ++k) { sa = mfma32(kfr[k], qf[k], sa); pa = mfma32(vfr[k], dof[k], pa); }
}
template <int KROW0>
__device__ __forceinline__ void dq_acc64(f32x16 (&dq_acc)[4], const char* Ks, const LaneOffsets& lo, bf16x8 dsf) {
#pragma unroll
  for (int db = 0; db < 2; ++db) dq_acc[db] = mfma32(frag_tr<KROW0>(Ks, lo, db), dsf, dq_acc[db]);
}
__device__ __forceinline__ void dq_tile64(f32x16 (&dq_acc)[4], const bf16x8 (&qf)[8], const bf16x8 (&dof)[8],
                                          const char* Ks, const char* Vs, const LaneOffsets& lo, int j0,
                                          int qrow, float c2, float lse2, float delta, int g32, bool masked) {
  bf16x8 dsf[4];
  f32x16 sa = zero16(), pa = zero16();
  dq_scores64<0>(sa, pa, qf, dof, Ks, Vs, lo);
  dq_ds<0>(sa, pa, dsf[0], dsf[1], j0, qrow, c2, lse2, delta, g32, masked);
  sa = zero16();
  pa = zero16();
  dq_scores64<32>(sa, pa, qf, dof, Ks, Vs, lo);
  dq_ds<32>(sa, pa, dsf[2], dsf[3], j0, qrow, c2, lse2, delta, g32, masked);
  dq_acc64<0>(dq_acc, Ks, lo, dsf[0]);
  dq_acc64<16>(dq_acc, Ks, lo, dsf[1]);
  dq_acc64<32>(dq_acc, Ks, lo, dsf[2]);
  dq_acc64<48>(dq_acc, Ks, lo, dsf[3]);
}

// DH = 64 (only with RAGGED): the head dimension is 64 and the products skip the zero half.
template <bool RAGGED, int DH = 128>
__global__ void __launch_bounds__(256, 2)
bwd_dq_bf16_kernel(KArgs a, int T, int il, int n_rest) {
  constexpr int BM = 128;
  __shared__ __attribute__((aligned(1024))) char smem[4 * kTileBytes];   // [stage][K,V]

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g32 = lane >> 5, l32 = lane & 31;

  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int y, rank;
  decode_slot(slot, T, il, y, rank);
  int qt = T - 1 - rank;
  const int hr = uni(y % a.r);
  int rest = uni(uni(y / a.r) * 8 + xcd);
  if (rest >= n_rest) return;
  const int NG = uni(a.N / a.G);
  const int gidx = uni(rest % NG); rest = uni(rest / NG);
  const int c = uni(rest % a.Hkv);
  const int b = uni(rest / a.Hkv);
  const int h = c * a.r + hr;

  const int s = uni(shift_of_head(a, h));
  Run run{gidx * a.G, a.G};                        // the causal run of this block (see the forward kernel)
  int split = uni(split_of_group(a, gidx, s));
  if constexpr (RAGGED) {
    if (!run_of_tile(a, gidx, s, BM, qt, run)) return;
    run.p0 = uni(run.p0); run.len = uni(run.len);
    split = run.len;
  }
  const int i0 = qt * BM;
  const int qw0 = i0 + w * 32;
  const int qrow = qw0 + l32;
  const int lo_w = uni(qw0 >= split ? split : 0);
  const int jt_first = uni((i0 >= split ? split : 0) / BN);
  const int jt_diag = i0 / BN;
  const float c2 = a.scale_log2;

  const char* kp = static_cast<const char*>(a.k);
  const char* vp = static_cast<const char*>(a.v);

  bf16x8 qf[8], dof[8];
  float lse2, delta;
  {
    const int tok = run_token(a, run, qrow, s);
    const bf16x8* qsrc = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(a.q) + row_off(a.sq, b, tok, h));
    const bf16x8* dsrc = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(a.dout) + row_off(a.so, b, tok, h));
#pragma unroll
    for (int st = 0; st < DH / 16; ++st) { qf[st] = qsrc[2 * st + g32]; dof[st] = dsrc[2 * st + g32]; }
    const size_t ro = ((size_t)b * a.H + h) * a.N + tok;
    lse2 = a.lse2[ro];
    delta = a.delta[ro];
  }

  const uint32_t smem_base = lds_addr(smem);
  const uint64_t k_row_bytes = (uint64_t)a.sk.t * 2, v_row_bytes = (uint64_t)a.sv.t * 2;
  const int st_row = 4 * w + (lane >> 4);
  const uint32_t st_chunk = (uint32_t)(((lane & 15) ^ swz(st_row)) << 4);
  // aligned staging: scalar base of the tile's 64-token run plus these per-lane offsets
  const uint32_t k_lane = (uint32_t)(st_row * k_row_bytes) + st_chunk;
  const uint32_t v_lane = (uint32_t)(st_row * v_row_bytes) + st_chunk;
  const uint64_t k_head = uni64(reinterpret_cast<uint64_t>(kp) + row_off(a.sk, b, 0, c) * 2);
  const uint64_t v_head = uni64(reinterpret_cast<uint64_t>(vp) + row_off(a.sv, b, 0, c) * 2);
  auto issue_tile = [&](int jt, int stage) {
    const uint32_t ks = smem_base + stage * 2 * kTileBytes + 4 * w * kRowBytes;
    if constexpr (!RAGGED) {
      const uint32_t tok0 = (uint32_t)token_of(run.p0 + jt * BN, s, a.N);   // an aligned tile never straddles the wrap
      const uint64_t kb = k_head + tok0 * k_row_bytes, vb = v_head + tok0 * v_row_bytes;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        dma16s(kb + p * 16 * k_row_bytes, k_lane, ks + 16 * p * kRowBytes);
        dma16s(vb + p * 16 * v_row_bytes, v_lane, ks + 16 * p * kRowBytes + kTileBytes);
      }
    } else {   // every row finds its own token; padding rows repeat the last row of the group
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int tok = run_token(a, run, jt * BN + 16 * p + st_row, s);
        if (DH == 128 || st_chunk < 2 * DH) {   // a 64-wide row fills the first eight chunks only
          dma16(kp + row_off(a.sk, b, tok, c) * 2 + st_chunk, ks + 16 * p * kRowBytes);
          dma16(vp + row_off(a.sv, b, tok, c) * 2 + st_chunk, ks + 16 * p * kRowBytes + kTileBytes);
        }
      }
    }
  };

  LaneOffsets lo;
  init_lane_offsets(lo, lane);
  f32x16 dq_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) dq_acc[db] = zero16();

  issue_tile(jt_first, 0);
  const int n_tiles = jt_diag + 2 - jt_first;
  // The stage is a compile-time constant of the body (the loop is unrolled by the number
  // of stages), so every LDS read is lane offset + immediate.
  auto body = [&](auto stage_c, int n) {
    constexpr int STAGE = decltype(stage_c)::value;
    const int jt = jt_first + n;
    wait_vmcnt0();
    __syncthreads();
    if (n + 1 < n_tiles) issue_tile(jt + 1, STAGE ^ 1);
    const int j0 = jt * BN;
    const char* Ks = smem + STAGE * 2 * kTileBytes;
    const char* Vs = Ks + kTileBytes;
    if (j0 > qw0 + 31 || j0 + BN - 1 < lo_w) return;   // wholly outside this wave's visible keys
    if constexpr (DH == 128)
      dq_tile(dq_acc, qf, dof, Ks, Vs, lo, j0, qrow, c2, lse2, delta, g32, j0 + BN - 1 > qw0);
    else
      dq_tile64(dq_acc, qf, dof, Ks, Vs, lo, j0, qrow, c2, lse2, delta, g32, j0 + BN - 1 > qw0);
  };
  for (int n = 0; n < n_tiles; n += 2) {
    body(std::integral_constant<int, 0>{}, n);
    if (n + 1 < n_tiles) body(std::integral_constant<int, 1>{}, n + 1);
  }
  __syncthreads();

  char* region = smem + w * (32 * kRowBytes);
  acc_to_lds(region, dq_acc, a.scale, l32, g32);
  __syncthreads();
  __bf16* dqp = static_cast<__bf16*>(a.dq);
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int row = it * 4 + (lane >> 4), ch = lane & 15;
    if (qw0 + row >= run.len || ch * 8 >= a.D) continue;   // padding row of a partial tile, padding of a narrow row
    const int tok = token_of(run.p0 + qw0 + row, s, a.N);
    *reinterpret_cast<uint4*>(dqp + row_off(a.sdq, b, tok, h) + ch * 8) =
        *reinterpret_cast<const uint4*>(region + tile_off(row, ch));
  }
}

}  // namespace

int launch_bwd_dkdv_bf16(const KArgs& a, hipStream_t st) {
  if (dkdv_split_applies(a)) return launch_bwd_dkdv_split_bf16(a, st);
  const int NG = a.N / a.G;
  const int ncls = a.mixed ? 2 : 1;
  const int T = a.ragged ? ragged_tiles(a, 128) : a.G / 128;
  const int n_rest = a.B * a.Hkv * ncls * NG;
  const int il = interleave_for(T, 32);   // 32 CUs per XCD, one workgroup each
  const int blocks = 8 * T * pad_to((n_rest + 7) / 8, il);
  if (a.D == 64)
    hipLaunchKernelGGL((bwd_dkdv_bf16_kernel<true, 64>), dim3(blocks), dim3(256), 0, st, a, ncls, T, il, n_rest);
  else if (a.ragged)
    hipLaunchKernelGGL(bwd_dkdv_bf16_kernel<true>, dim3(blocks), dim3(256), 0, st, a, ncls, T, il, n_rest);
  else
    hipLaunchKernelGGL(bwd_dkdv_bf16_kernel<false>, dim3(blocks), dim3(256), 0, st, a, ncls, T, il, n_rest);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_bwd_dq_bf16(const KArgs& a, hipStream_t st) {
  const int NG = a.N / a.G;
  const int T = a.ragged ? ragged_tiles(a, 128) : a.G / 128;
  const int n_rest = a.B * a.Hkv * NG;
  const int il = interleave_for(T, 64);   // 32 CUs per XCD, two workgroups each
  const int blocks = 8 * T * pad_to(a.r * ((n_rest + 7) / 8), il);
  if (a.D == 64)
    hipLaunchKernelGGL((bwd_dq_bf16_kernel<true, 64>), dim3(blocks), dim3(256), 0, st, a, T, il, n_rest);
  else if (a.ragged)
    hipLaunchKernelGGL(bwd_dq_bf16_kernel<true>, dim3(blocks), dim3(256), 0, st, a, T, il, n_rest);
  else
    hipLaunchKernelGGL(bwd_dq_bf16_kernel<false>, dim3(blocks), dim3(256), 0, st, a, T, il, n_rest);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace s2
