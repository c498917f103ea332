// bf16 S2-Attn forward for gfx950: tiled online-softmax attention inside each group
// of LongLoRA Section 3.2, with the shift of Algorithm 1 folded into row addresses.
//
// One workgroup (4 waves) owns 128 consecutive query rows of one (batch, head, group)
// in the head's rolled frame; a wave owns 32 of them.  It walks the 64-key tiles of
// the same group up to the diagonal.  Per tile and wave:
//   S^T = K Q^T        A = K rows from LDS (row-major fragments), B = Q^T in registers
//   online softmax     queries are lane-indexed, keys register-indexed, so row max and
//                      row sum are in-lane reductions plus one exchange with lane^32;
//                      the running maximum is only raised (and O rescaled) when it
//                      grows by more than 2^8, which keeps exp2 arguments <= 8
//   O^T += V^T P^T     A = V^T through transposing LDS reads, B = P^T straight from the
//                      S^T accumulators (no cross-lane movement)
// K/V tiles go global -> LDS directly (global_load_lds, 16 bytes per lane) into two
// stages, one barrier per tile.  The output tile is transposed through LDS and stored
// with 16-byte coalesced writes at the un-rolled token rows.
#include "s2attn_bf16_common.h"
#include "s2attn_device.h"
#include "s2attn_launch.h"

namespace s2 {
namespace {

constexpr int BN = 64;                       // keys per tile
constexpr int kTileBytes = BN * kRowBytes;   // 16 KB
constexpr float kRescaleThreshold = 8.f;     // log2 units

struct FwdState {
  f32x16 o_acc[4];
  float m_run;    // running row maximum (raw score units), shared by lanes l and l^32
  float l_run;    // this lane's part of the running row sum
};

// O^T += V^T P^T for the 16 keys starting at tile row KROW0.  DH: head dimension the products
// run over (128, or 64 when the upper half of every tile row is zero padding).
template <int KROW0, int DH = 128>
__device__ __forceinline__ void pv_step(FwdState& st, const char* Vs, const LaneOffsets& lo, bf16x8 pf) {
  bf16x8 vf[DH / 32];
#pragma unroll
  for (int db = 0; db < DH / 32; ++db) vf[db] = frag_tr<KROW0>(Vs, lo, db);
#pragma unroll
  for (int db = 0; db < DH / 32; ++db) st.o_acc[db] = mfma32(vf[db], pf, st.o_acc[db]);
}

// S^T = K Q^T of one 64-key tile for one wave (32 queries): two 32-key blocks.
// `masked` is wave-uniform: the tile touches the diagonal of this wave's rows.
template <int DH = 128>
__device__ __forceinline__ void fwd_scores(f32x16& s0, f32x16& s1, const bf16x8 (&qf)[8], const char* Ks,
                                           const LaneOffsets& lo, int j0, int qrow, int g32, bool masked) {
  s0 = zero16();
  s1 = zero16();
  bf16x8 ka[4], kb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ka[i] = frag_rm<0>(Ks, lo, i);
    kb[i] = frag_rm<32>(Ks, lo, i);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    s0 = mfma32(ka[i], qf[i], s0);
    s1 = mfma32(kb[i], qf[i], s1);
  }
  if constexpr (DH == 128) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ka[i] = frag_rm<0>(Ks, lo, i + 4);
      kb[i] = frag_rm<32>(Ks, lo, i + 4);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s0 = mfma32(ka[i], qf[i + 4], s0);
      s1 = mfma32(kb[i], qf[i + 4], s1);
    }
  }
  if (masked) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = j0 + 8 * (v >> 2) + 4 * g32 + (v & 3);
      if (key > qrow) s0[v] = -INFINITY;
      if (key + 32 > qrow) s1[v] = -INFINITY;
    }
  }
}

// Online softmax of the tile: updates the running maximum lazily, accumulates the row
// sum and packs the probabilities as the four 16-key B operands of the PV product.
__device__ __forceinline__ void fwd_softmax(FwdState& st, f32x16& s0, f32x16& s1, float c2, bf16x8 (&pf)[4]) {
  // two independent three-input maximum chains
  float ma = fmaxf(s0[0], s0[1]), mb = fmaxf(s1[0], s1[1]);
#pragma unroll
  for (int v = 2; v < 16; v += 2) {
    ma = fmaxf(fmaxf(ma, s0[v]), s0[v + 1]);
    mb = fmaxf(fmaxf(mb, s1[v]), s1[v + 1]);
  }
  const float mx = max_halves(fmaxf(ma, mb));
  if (__builtin_amdgcn_ballot_w64(mx * c2 > st.m_run * c2 + kRescaleThreshold) != 0) {
    const float m_new = fmaxf(st.m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f((st.m_run - m_new) * c2);
    st.m_run = m_new;
    st.l_run *= alpha;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) st.o_acc[db][v] *= alpha;
  }
  const float mc = st.m_run * c2;
  float ra = 0.f, rb = 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    s0[v] = __builtin_amdgcn_exp2f(fmaf(s0[v], c2, -mc));
    s1[v] = __builtin_amdgcn_exp2f(fmaf(s1[v], c2, -mc));
    ra += s0[v];
    rb += s1[v];
  }
  st.l_run += ra + rb;
  pf[0] = pack8(s0[0], s0[1], s0[2], s0[3], s0[4], s0[5], s0[6], s0[7]);
  pf[1] = pack8(s0[8], s0[9], s0[10], s0[11], s0[12], s0[13], s0[14], s0[15]);
  pf[2] = pack8(s1[0], s1[1], s1[2], s1[3], s1[4], s1[5], s1[6], s1[7]);
  pf[3] = pack8(s1[8], s1[9], s1[10], s1[11], s1[12], s1[13], s1[14], s1[15]);
}

// O^T += V^T P^T for the whole 64-key tile.
template <int DH = 128>
__device__ __forceinline__ void fwd_pv(FwdState& st, const char* Vs, const LaneOffsets& lo, const bf16x8 (&pf)[4]) {
  pv_step<0, DH>(st, Vs, lo, pf[0]);
  pv_step<16, DH>(st, Vs, lo, pf[1]);
  pv_step<32, DH>(st, Vs, lo, pf[2]);
  pv_step<48, DH>(st, Vs, lo, pf[3]);
}

template <int DH = 128>
__device__ __forceinline__ void fwd_tile(FwdState& st, const bf16x8 (&qf)[8], const char* Ks, const char* Vs,
                                         const LaneOffsets& lo, int j0, int qrow, float c2, int g32, bool masked) {
  f32x16 s0, s1;
  bf16x8 pf[4];
  fwd_scores<DH>(s0, s1, qf, Ks, lo, j0, qrow, g32, masked);
  fwd_softmax(st, s0, s1, c2, pf);
  fwd_pv<DH>(st, Vs, lo, pf);
}

// Normalises a wave's 32 x 128 output block, transposes it through the wave's private
// 8 KB LDS region and stores it (and lse) at the un-rolled token rows.  Contains one
// workgroup barrier between the LDS writes and reads.
__device__ __forceinline__ void fwd_epilogue(const KArgs& a, FwdState& st, char* Os, int b, int h, const Run& run, int s,
                                             int qw0, float c2, int lane, int l32, int g32) {
  __bf16* op = static_cast<__bf16*>(a.o);
  const float l_tot = sum_halves(st.l_run);
  const float inv = 1.f / l_tot;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) {
      const bf16x4 pk = pack4(st.o_acc[db][4 * vv] * inv, st.o_acc[db][4 * vv + 1] * inv,
                              st.o_acc[db][4 * vv + 2] * inv, st.o_acc[db][4 * vv + 3] * inv);
      *reinterpret_cast<bf16x4*>(Os + tile_off(l32, 4 * db + vv) + 8 * g32) = pk;
    }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int row = it * 4 + (lane >> 4), ch = lane & 15;
    const uint4 val = *reinterpret_cast<const uint4*>(Os + tile_off(row, ch));
    if (qw0 + row < run.len && ch * 8 < a.D) {   // rows past the end of the run are padding of a partial tile
      const int tok = token_of(run.p0 + qw0 + row, s, a.N);
      *reinterpret_cast<uint4*>(op + row_off(a.so, b, tok, h) + ch * 8) = val;
    }
  }
  if (g32 == 0 && qw0 + l32 < run.len) {
    const int tok = token_of(run.p0 + qw0 + l32, s, a.N);
    a.lse[((size_t)b * a.H + h) * a.N + tok] = (st.m_run * c2 + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }
}

// RAGGED: G is not a multiple of 128, the shift not of 64 or a Variant 2 split not of 128 --
// tiles may be partial and the wrap point may fall inside one, so every staged row finds
// its own token, and the two halves of a split wrap-around group run as causal runs of
// their own (run_of_tile).
// DH = 64 (only with RAGGED): the head dimension is 64 and the products skip the zero half.
template <bool RAGGED, int DH = 128>
__global__ void __launch_bounds__(256, 2)
fwd_bf16_kernel(KArgs a, int T, int il, int n_rest) {
  constexpr int BM = 128;
  __shared__ __attribute__((aligned(1024))) char smem[4 * kTileBytes];   // [stage][K,V]

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g32 = lane >> 5, l32 = lane & 31;

  // ---- block -> (batch, head, group, query tile).  Consecutive block ids go to
  // different XCDs, so the id is split as (xcd, slot): every XCD walks its own
  // sequence of (batch, kv head, group) triples, all query heads of the kv head and
  // all query tiles (heaviest first) of a triple back to back, so that the K/V of a
  // group stay in that XCD's L2 while they are being re-read.
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
  // the causal run this block works in and the first row of the other block of a split
  // wrap-around group inside it (aligned kernels skip whole tiles at `split`; the ragged
  // ones run the two blocks as runs of their own and see no split)
  Run run{gidx * a.G, a.G};
  int split = uni(split_of_group(a, gidx, s));
  if constexpr (RAGGED) {
    if (!run_of_tile(a, gidx, s, BM, qt, run)) return;
    run.p0 = uni(run.p0); run.len = uni(run.len);
    split = run.len;
  }
  const int i0 = qt * BM;
  const int qw0 = i0 + w * 32;                      // first query row of this wave
  const int qrow = qw0 + l32;
  const int lo_w = uni(qw0 >= split ? split : 0);        // first key visible to this wave
  const int jt_first = uni((i0 >= split ? split : 0) / BN);
  const int jt_diag = i0 / BN;                      // tiles jt_diag, jt_diag + 1 touch the diagonal
  const float c2 = a.scale_log2;

  const __bf16* qp = static_cast<const __bf16*>(a.q);
  const char* kp = static_cast<const char*>(a.k);
  const char* vp = static_cast<const char*>(a.v);

  // ---- Q^T fragments of this wave, straight from global memory
  bf16x8 qf[8];
  {
    const int tok = run_token(a, run, qrow, s);
    const bf16x8* src = reinterpret_cast<const bf16x8*>(qp + row_off(a.sq, b, tok, h));
#pragma unroll
    for (int st = 0; st < DH / 16; ++st) qf[st] = src[2 * st + g32];
  }

  // ---- K/V staging, global -> LDS: wave w, pass p fills tile rows 16p + 4w .. +3
  // (1 KB contiguous in LDS); lane i lands on physical chunk i%16 of row i/16 and
  // therefore fetches the logical chunk that the swizzle places there.
  const int st_row = 4 * w + (lane >> 4);
  const uint64_t k_row_bytes = (uint64_t)a.sk.t * 2, v_row_bytes = (uint64_t)a.sv.t * 2;
  const uint32_t smem_base = lds_addr(smem);
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
  FwdState st;
  st.m_run = -INFINITY;
  st.l_run = 0.f;
#pragma unroll
  for (int db = 0; db < 4; ++db) st.o_acc[db] = zero16();

  issue_tile(jt_first, 0);
  const int n_tiles = jt_diag + 2 - jt_first;
  for (int n = 0; n < n_tiles; ++n) {
    const int jt = jt_first + n;
    const int stage = n & 1;
    wait_vmcnt0();                        // this wave's part of tile jt has landed
    __syncthreads();                      // everyone's part has landed; everyone left tile jt-1
    if (n + 1 < n_tiles) issue_tile(jt + 1, stage ^ 1);
    const int j0 = jt * BN;
    const char* Ks = smem + stage * 2 * kTileBytes;
    const char* Vs = Ks + kTileBytes;
    // this wave's rows see keys [lo_w, row]: skip tiles wholly outside (beyond the
    // diagonal, or, under Variant 2, in the other block of the wrap group)
    if (j0 > qw0 + 31 || j0 + BN - 1 < lo_w) continue;
    fwd_tile<DH>(st, qf, Ks, Vs, lo, j0, qrow, c2, g32, j0 + BN - 1 > qw0);
  }
  __syncthreads();

  // ---- epilogue: normalise, transpose through LDS, store at un-rolled token rows
  fwd_epilogue(a, st, smem + w * (32 * kRowBytes), b, h, run, s, qw0, c2, lane, l32, g32);
}

// ---- the matrix block of the eight-wave kernel as 8 steps of 4 MFMAs, each fed by 4
// operand fragments.  Steps 0-3: O^T += V^T P^T for keys 16k .. 16k+15 of the current
// tile; steps 4-7: S^T += K Q^T over d = 32(k-4) .. +31 of the next tile.
template <int STEP>
__device__ __forceinline__ void pp_load(bf16x8 (&buf)[4], const char* Vs_cur, const char* Ks_nxt, const LaneOffsets& lo) {
  if constexpr (STEP < 4) {
#pragma unroll
    for (int db = 0; db < 4; ++db) buf[db] = frag_tr<16 * STEP>(Vs_cur, lo, db);
  } else {
    constexpr int J = STEP - 4;
    buf[0] = frag_rm<0>(Ks_nxt, lo, 2 * J);
    buf[1] = frag_rm<32>(Ks_nxt, lo, 2 * J);
    buf[2] = frag_rm<0>(Ks_nxt, lo, 2 * J + 1);
    buf[3] = frag_rm<32>(Ks_nxt, lo, 2 * J + 1);
  }
}

template <int STEP>
__device__ __forceinline__ void pp_mma(const bf16x8 (&buf)[4], FwdState& st, const bf16x8 (&pf)[4],
                                       const bf16x8 (&qf)[8], f32x16& s0, f32x16& s1) {
  if constexpr (STEP < 4) {
#pragma unroll
    for (int db = 0; db < 4; ++db) st.o_acc[db] = mfma32(buf[db], pf[STEP], st.o_acc[db]);
  } else {
    constexpr int J = STEP - 4;
    s0 = mfma32(buf[0], qf[2 * J], s0);
    s1 = mfma32(buf[1], qf[2 * J], s1);
    s0 = mfma32(buf[2], qf[2 * J + 1], s0);
    s1 = mfma32(buf[3], qf[2 * J + 1], s1);
  }
}

__device__ __forceinline__ void mask_scores(f32x16& s0, f32x16& s1, int j0, int qrow, int g32) {
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int key = j0 + 8 * (v >> 2) + 4 * g32 + (v & 3);
    if (key > qrow) s0[v] = -INFINITY;
    if (key + 32 > qrow) s1[v] = -INFINITY;
  }
}

// ---------------------------------------------------------------------------
// Eight-wave variant (G a multiple of 256): a workgroup owns 256 query rows and keeps
// three K/V stages in LDS, one workgroup per CU, two waves per SIMD.  Each wave runs
// the tile loop software-pipelined across tiles: the matrix block of an iteration is
// P(n) V(n) followed by S(n+1) = K(n+1) Q^T, the vector block is the softmax of one
// tile.  Waves 0-3 run the vector block after the matrix block, waves 4-7 before it,
// so the two waves that share a SIMD alternate between the matrix and vector units
// instead of competing for them ("ping-pong"), with a single barrier per tile.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(512, 1)
fwd_bf16_pp_kernel(KArgs a, int T, int il, int n_rest) {
  constexpr int BM = 256;
  constexpr int kStageBytes = 2 * kTileBytes;
  __shared__ __attribute__((aligned(1024))) char smem[3 * kStageBytes];   // [stage][K,V]

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g32 = lane >> 5, l32 = lane & 31;
  const int grp = w >> 2;

  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int y, rank;
  decode_slot(slot, T, il, y, rank);
  const int qt = T - 1 - rank;
  const int hr = uni(y % a.r);
  int rest = uni(uni(y / a.r) * 8 + xcd);
  if (rest >= n_rest) return;
  const int NG = uni(a.N / a.G);
  const int gidx = uni(rest % NG); rest = uni(rest / NG);
  const int c = uni(rest % a.Hkv);
  const int b = uni(rest / a.Hkv);
  const int h = c * a.r + hr;

  const int s = uni(shift_of_head(a, h));
  const int split = uni(split_of_group(a, gidx, s));
  const int i0 = qt * BM;
  const int qw0 = i0 + w * 32;
  const int qrow = qw0 + l32;
  const int jt_first = uni((i0 >= split ? split : 0) / BN);     // first tile any wave needs
  const int nt = uni((i0 + BM - 1) / BN - jt_first + 1);   // tiles the workgroup walks
  // this wave's own tile range, relative to jt_first
  const int n_lo = uni((qw0 >= split ? split : 0) / BN - jt_first);
  const int n_hi = uni((qw0 + 31) / BN - jt_first);
  const float c2 = a.scale_log2;

  const __bf16* qp = static_cast<const __bf16*>(a.q);
  const char* kp = static_cast<const char*>(a.k);
  const char* vp = static_cast<const char*>(a.v);

  bf16x8 qf[8];
  {
    const int tok = token_of(gidx * a.G + qrow, s, a.N);
    const bf16x8* src = reinterpret_cast<const bf16x8*>(qp + row_off(a.sq, b, tok, h));
#pragma unroll
    for (int st = 0; st < 8; ++st) qf[st] = src[2 * st + g32];
  }

  // staging: wave w, pass p fills tile rows 32p + 4w .. +3 of K and of V.  A tile is a
  // contiguous run of 64 tokens, so its address is a scalar (head base + first token) plus a
  // per-lane offset (row within the pass, swizzled chunk) that never changes.
  const int st_row = 4 * w + (lane >> 4);
  const uint64_t k_row_bytes = (uint64_t)a.sk.t * 2, v_row_bytes = (uint64_t)a.sv.t * 2;
  const uint32_t smem_base = lds_addr(smem);
  const uint32_t st_chunk = (uint32_t)(((lane & 15) ^ swz(st_row)) << 4);
  const uint32_t k_lane = (uint32_t)(st_row * k_row_bytes) + st_chunk;
  const uint32_t v_lane = (uint32_t)(st_row * v_row_bytes) + st_chunk;
  const uint64_t k_head = uni64(reinterpret_cast<uint64_t>(kp) + row_off(a.sk, b, 0, c) * 2);
  const uint64_t v_head = uni64(reinterpret_cast<uint64_t>(vp) + row_off(a.sv, b, 0, c) * 2);
  auto issue_tile = [&](int n, int stage) {
    const uint32_t tok0 = (uint32_t)token_of(gidx * a.G + (jt_first + n) * BN, s, a.N);
    const uint64_t kb = k_head + tok0 * k_row_bytes, vb = v_head + tok0 * v_row_bytes;
    const uint32_t ks = smem_base + stage * kStageBytes + 4 * w * kRowBytes;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      dma16s(kb + p * 32 * k_row_bytes, k_lane, ks + 32 * p * kRowBytes);
      dma16s(vb + p * 32 * v_row_bytes, v_lane, ks + 32 * p * kRowBytes + kTileBytes);
    }
  };

  LaneOffsets lo;
  init_lane_offsets(lo, lane);
  FwdState st;
  st.m_run = -INFINITY;
  st.l_run = 0.f;
#pragma unroll
  for (int db = 0; db < 4; ++db) st.o_acc[db] = zero16();
  f32x16 s0, s1;       // scores of the tile whose softmax is pending
  bf16x8 pf[4];        // probabilities of the tile whose PV product is pending
  bf16x8 ring[4][4];   // operand fragments of steps k, k+1, k+2 (slot = step mod 4)

  // ---- prologue: tiles 0 and 1 in flight, scores of tile 0
  issue_tile(0, 0);
  if (nt > 1) {
    issue_tile(1, 1);
    __builtin_amdgcn_s_waitcnt(0x0F74);   // vmcnt(4): tile 0 has landed, tile 1 may be in flight
  } else {
    wait_vmcnt0();
  }
  __syncthreads();
  if (n_lo <= 0 && 0 <= n_hi) {
    fwd_scores(s0, s1, qf, smem, lo, jt_first * BN, qrow, g32, jt_first * BN + BN - 1 > qw0);
    if (grp == 0) fwd_softmax(st, s0, s1, c2, pf);
    pp_load<0>(ring[0], smem + kTileBytes, nullptr, lo);     // first two steps of P(0) V(0)
    pp_load<1>(ring[1], smem + kTileBytes, nullptr, lo);
  }

  int st_cur = 0, st_nxt = 1, st_free = 2;   // stages of tile n, tile n+1, and the free one
  for (int n = 0; n < nt; ++n) {
    wait_vmcnt0();        // this wave's part of tile n+1 has landed
    __syncthreads();      // all of tile n+1 has landed; every wave has left tile n-1
    if (n + 2 < nt) issue_tile(n + 2, st_free);
    const bool act = n_lo <= n && n <= n_hi;
    const bool act_next = n + 1 < nt && n_lo <= n + 1 && n + 1 <= n_hi;
    const char* Vs_cur = smem + st_cur * kStageBytes + kTileBytes;
    const char* Ks_nxt = smem + st_nxt * kStageBytes;
    const char* Vs_nxt = Ks_nxt + kTileBytes;
    if (grp == 1 && act) fwd_softmax(st, s0, s1, c2, pf);
    // Every step issues the LDS reads of the step two ahead, then its own four MFMAs.  The
    // matrix block runs at raised priority so that it is not starved by the vector work of
    // the wave it shares the SIMD with.
    __builtin_amdgcn_s_setprio(1);
    if (act) {
      pp_load<2>(ring[2], Vs_cur, Ks_nxt, lo);
      pp_mma<0>(ring[0], st, pf, qf, s0, s1);
      __builtin_amdgcn_sched_barrier(0);
      pp_load<3>(ring[3], Vs_cur, Ks_nxt, lo);
      pp_mma<1>(ring[1], st, pf, qf, s0, s1);
      __builtin_amdgcn_sched_barrier(0);
      if (act_next) pp_load<4>(ring[0], Vs_cur, Ks_nxt, lo);
      pp_mma<2>(ring[2], st, pf, qf, s0, s1);
      __builtin_amdgcn_sched_barrier(0);
      if (act_next) pp_load<5>(ring[1], Vs_cur, Ks_nxt, lo);
      pp_mma<3>(ring[3], st, pf, qf, s0, s1);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (act_next) {
      if (!act) {   // this wave's first tile: nothing was prefetched
        pp_load<4>(ring[0], Vs_cur, Ks_nxt, lo);
        pp_load<5>(ring[1], Vs_cur, Ks_nxt, lo);
      }
      s0 = zero16();
      s1 = zero16();
      pp_load<6>(ring[2], Vs_cur, Ks_nxt, lo);
      pp_mma<4>(ring[0], st, pf, qf, s0, s1);
      __builtin_amdgcn_sched_barrier(0);
      pp_load<7>(ring[3], Vs_cur, Ks_nxt, lo);
      pp_mma<5>(ring[1], st, pf, qf, s0, s1);
      __builtin_amdgcn_sched_barrier(0);
      pp_load<0>(ring[0], Vs_nxt, nullptr, lo);     // first two steps of the next iteration
      pp_mma<6>(ring[2], st, pf, qf, s0, s1);
      __builtin_amdgcn_sched_barrier(0);
      pp_load<1>(ring[1], Vs_nxt, nullptr, lo);
      pp_mma<7>(ring[3], st, pf, qf, s0, s1);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(0);
      const int j0 = (jt_first + n + 1) * BN;
      if (j0 + BN - 1 > qw0) mask_scores(s0, s1, j0, qrow, g32);
      if (grp == 0) fwd_softmax(st, s0, s1, c2, pf);
    }
    __builtin_amdgcn_s_setprio(0);
    const int t = st_cur; st_cur = st_nxt; st_nxt = st_free; st_free = t;
  }
  __syncthreads();
  fwd_epilogue(a, st, smem + w * (32 * kRowBytes), b, h, Run{gidx * a.G, a.G}, s, qw0, c2, lane, l32, g32);
}

}  // namespace

int launch_fwd_bf16(const KArgs& a, hipStream_t st) {
  const int n_groups = a.B * a.Hkv * (a.N / a.G);
  // groups of 2048 tokens or more: the eight-wave kernel; shorter tile sequences run a little
  // faster (4-9 % at G = 512 ... 1024) with two independent four-wave workgroups per CU, whose
  // prologues and epilogues overlap
  if (a.G % 256 == 0 && a.G >= 2048 && !a.ragged) {
    const int T = a.G / 256;
    const int il = interleave_for(T, 32);   // 32 CUs per XCD, one workgroup each
    const int blocks = 8 * T * pad_to(a.r * ((n_groups + 7) / 8), il);
    hipLaunchKernelGGL(fwd_bf16_pp_kernel, dim3(blocks), dim3(512), 0, st, a, T, il, n_groups);
    return hipGetLastError() == hipSuccess ? 0 : -1;
  }
  const int T = a.ragged ? ragged_tiles(a, 128) : a.G / 128;
  const int n_rest = a.B * a.Hkv * (a.N / a.G);
  const int il = interleave_for(T, 64);   // 32 CUs per XCD, two workgroups each
  const int blocks = 8 * T * pad_to(a.r * ((n_rest + 7) / 8), il);
  if (a.D == 64)
    hipLaunchKernelGGL((fwd_bf16_kernel<true, 64>), dim3(blocks), dim3(256), 0, st, a, T, il, n_rest);
  else if (a.ragged)
    hipLaunchKernelGGL(fwd_bf16_kernel<true>, dim3(blocks), dim3(256), 0, st, a, T, il, n_rest);
  else
    hipLaunchKernelGGL(fwd_bf16_kernel<false>, dim3(blocks), dim3(256), 0, st, a, T, il, n_rest);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace s2
