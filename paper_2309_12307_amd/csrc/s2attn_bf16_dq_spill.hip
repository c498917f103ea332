// bf16 S2-Attn backward, dQ from stored dS (gfx950).  Tile-aligned shapes only: the dK/dV
// kernel of s2attn_bf16_dkdv_split.hip has stored dS = P * (dP - delta) of every tile it
// visited (layout: s2attn_device.h), so dQ = scale * dS K is a plain product here, with
// neither the scores nor the softmax recomputed: 2 D flops per (query, key) pair instead of
// the 6 D of the recomputing dQ kernel.  The kernel is bound by reading dS once from HBM
// (2 bytes per pair); K tiles are re-read from L2 as in the other kernels.
//
// A workgroup (4 waves, one per CU) owns 128 query rows of one (batch, head, group) and walks
// the 64-key half tiles up to the diagonal.  Per step, dS^T (64 keys x 128 queries) and K
// (64 keys x 128) go global -> LDS; both are read back through transposing loads, keys being
// the contraction index: dQ^T += K^T dS^T with a wave's 32 queries on lanes.  The columns of
// a dS tile are queries in the permuted order of the blobs, so a wave's lane holds query
// ds_col_query(lane) of its 32; the epilogue stores rows accordingly.  Masked entries of the
// diagonal tiles were stored as zeros, so no mask is applied here.
#include <type_traits>

#include "s2attn_bf16_common.h"
#include "s2attn_device.h"
#include "s2attn_launch.h"

namespace s2 {
namespace {

constexpr int BK = 64;                        // keys per step
constexpr int kTileBytes = BK * kRowBytes;    // 16 KB: K tile, and dS^T tile of 128 queries
constexpr int kStages = 5;                    // LDS stages of [K, dS^T]; 160 KB in all
constexpr int kAhead = kStages - 1;           // steps whose loads are in flight ahead of the one computed

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding: vmcnt bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

__global__ void __launch_bounds__(256, 1)
bwd_dq_spill_kernel(KArgs a, int T, int il, int n_rest) {
  constexpr int BM = 128;
  __shared__ __attribute__((aligned(1024))) char smem[kStages * 2 * kTileBytes];   // [stage][K, dS^T]

  const int tid = threadIdx.x, lane = tid & 63, w = uni(tid >> 6);
  const int g32 = lane >> 5, l32 = lane & 31;

  // block -> (batch, head, group, query tile), as in the other kernels: every XCD walks its
  // own (batch, kv head, group) triples, heaviest query tiles first
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int y, rank;
  decode_slot(slot, T, il, y, rank);
  const int qt = T - 1 - rank;
  const int hr = uni(y % a.r);
  int rest = uni(uni(y / a.r) * 8 + xcd);
  if (rest >= n_rest) return;
  const int NG = uni(a.N / a.G);
  const int gidx = uni(rest % NG); rest = uni(rest / NG);
  const int c = uni(a.c_begin + rest % a.c_count);
  const int b = uni(rest / a.c_count);
  const int h = c * a.r + hr;

  const int s = uni(shift_of_head(a, h));
  const int split = uni(split_of_group(a, gidx, s));   // Variant 2: a multiple of 128 here
  const int i0 = qt * BM;
  const int qw0 = i0 + w * 32;
  const int jt_first = uni((i0 >= split ? split : 0) / 128);   // first 128-key tile with visible keys
  const int n_steps = 2 * (qt - jt_first + 1);

  // ---- staging.  Wave w, pass p fills tile rows 16p + 4w .. +3 of both tiles; lane i lands on
  // physical chunk i % 16 of its row and fetches the logical chunk the swizzle puts there.
  const uint32_t smem_base = lds_addr(smem);
  const int st_row = 4 * w + (lane >> 4);
  const int st_chunk = (lane & 15) ^ swz(st_row);
  // K: a tile is a contiguous run of 64 tokens
  const uint64_t k_row_bytes = (uint64_t)a.sk.t * 2;
  const uint32_t k_lane = (uint32_t)(st_row * k_row_bytes) + (uint32_t)(st_chunk << 4);
  const uint64_t k_head = uni64(reinterpret_cast<uint64_t>(a.k) + row_off(a.sk, b, 0, c) * 2);
  // dS^T: logical chunks 0-7 of a key's row come from the blob of the first 64 queries, 8-15
  // from that of the second (the next blob of the same key tile); chunk 2 f + g of key k is
  // the 16 bytes that lane 32 g + k % 32 of key block k / 32 stored from its operand f
  const uint32_t ds_lane = (uint32_t)((st_chunk >> 3) * kDsBlobBytes + ((st_chunk >> 1) & 3) * 1024 +
                                      (st_chunk & 1) * 512 + st_row * 16);
  const long long per_group = ds_blobs_per_group(T);
  const uint64_t ds_group = uni64(reinterpret_cast<uint64_t>(a.ds_spill) +
      (uint64_t)(((long long)(b * a.c_count * a.r + (h - a.c_begin * a.r)) * NG + gidx) * per_group) * kDsBlobBytes);
  auto issue_step = [&](int n, int stage) {
    const int jt = jt_first + (n >> 1), half = n & 1;
    const uint32_t tok0 = (uint32_t)token_of(gidx * a.G + jt * 128 + half * BK, s, a.N);
    const uint64_t kb = k_head + tok0 * k_row_bytes;
    const uint64_t db = ds_group + (uint64_t)ds_blob_index(T, jt, 2 * (qt - jt)) * kDsBlobBytes + half * 8192;
    const uint32_t ks = smem_base + stage * 2 * kTileBytes + 4 * w * kRowBytes;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      dma16s(kb + p * 16 * k_row_bytes, k_lane, ks + 16 * p * kRowBytes);
      // keys 16 p .. 16 p + 15 of the half tile: key block p / 2, lanes 16 (p % 2) ...
      dma16s(db + (p >> 1) * 4096 + (p & 1) * 256, ds_lane, ks + 16 * p * kRowBytes + kTileBytes);
    }
  };

  LaneOffsets lo;
  init_lane_offsets(lo, lane);
  // transposed fragment of this wave's column block of the dS^T tile: the two byte offsets of
  // init_lane_offsets for column block w, computed here because w is not a compile-time index
  int ds_tr[2];
  {
    const int L = lane & 15, row = 4 * g32 + (L >> 2);
    const int col = 32 * w + (lane & 16) + 4 * (L & 3);
    ds_tr[0] = row * kRowBytes + (((col >> 3) ^ swz(row)) << 4) + (col & 7) * 2;
    ds_tr[1] = (row + 8) * kRowBytes + (((col >> 3) ^ swz(row + 8)) << 4) + (col & 7) * 2;
  }
  auto ds_frag = [&](const char* tile, int krow0) {
    const bf16x4 a0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(S2_LDS(bf16x4, tile + ds_tr[0] + krow0 * kRowBytes));
    const bf16x4 a1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(S2_LDS(bf16x4, tile + ds_tr[1] + krow0 * kRowBytes));
    return __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
  };
  f32x16 dq_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) dq_acc[db] = zero16();

  // The kernel is bound by the latency and bandwidth of the dS reads, so the loads of kAhead
  // steps are kept in flight: loads complete in issue order, and each step issues 8 per wave.
#pragma unroll
  for (int n = 0; n < kAhead; ++n)
    if (n < n_steps) issue_step(n, n);
  auto body = [&](auto stage_c, int n) {
    constexpr int STAGE = decltype(stage_c)::value;
    if (n >= n_steps) return;
    if (n + kAhead <= n_steps) wait_vmcnt<(kAhead - 1) * 8>(); else wait_vmcnt0();
    __syncthreads();      // step n has landed for every wave; everyone has left step n - 1
    if (n + kAhead < n_steps) issue_step(n + kAhead, (STAGE + kAhead) % kStages);
    const char* Ks = smem + STAGE * 2 * kTileBytes;
    const char* Ds = Ks + kTileBytes;
    const int k0 = (jt_first + (n >> 1)) * 128 + (n & 1) * BK;
    if (k0 > qw0 + 31) return;   // keys after all of this wave's queries: the stored dS is zero
    // four k-steps of 16 keys: one dS^T fragment (this wave's 32 queries) against four K^T fragments
    bf16x8 fa[4], fb[4], dsa, dsb;
#pragma unroll
    for (int db = 0; db < 4; ++db) fa[db] = frag_tr<0>(Ks, lo, db);
    dsa = ds_frag(Ds, 0);
    __builtin_amdgcn_sched_barrier(0);
#define S2_STEP(T16, CUR, DSC, NXT, DSN)                                        \
    if (T16 < 48) {                                                             \
      _Pragma("unroll") for (int db = 0; db < 4; ++db) NXT[db] = frag_tr<(T16 < 48 ? T16 + 16 : 0)>(Ks, lo, db); \
      DSN = ds_frag(Ds, T16 < 48 ? T16 + 16 : 0);                               \
    }                                                                           \
    _Pragma("unroll") for (int db = 0; db < 4; ++db) dq_acc[db] = mfma32(CUR[db], DSC, dq_acc[db]); \
    __builtin_amdgcn_sched_barrier(0)
    S2_STEP(0, fa, dsa, fb, dsb);
    S2_STEP(16, fb, dsb, fa, dsa);
    S2_STEP(32, fa, dsa, fb, dsb);
    S2_STEP(48, fb, dsb, fa, dsa);
#undef S2_STEP
  };
  for (int n = 0; n < n_steps; n += kStages) {
    body(std::integral_constant<int, 0>{}, n);
    body(std::integral_constant<int, 1>{}, n + 1);
    body(std::integral_constant<int, 2>{}, n + 2);
    body(std::integral_constant<int, 3>{}, n + 3);
    body(std::integral_constant<int, 4>{}, n + 4);
  }
  __syncthreads();

  // ---- store: lane l of the wave holds query 32 w + ds_col_query(l) of the tile
  char* region = smem + w * (32 * kRowBytes);
  acc_to_lds(region, dq_acc, a.scale, l32, g32);
  __syncthreads();
  __bf16* dqp = static_cast<__bf16*>(a.dq);
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int row = it * 4 + (lane >> 4), ch = lane & 15;
    const int tok = token_of(gidx * a.G + qw0 + ds_col_query(row), s, a.N);
    *reinterpret_cast<uint4*>(dqp + row_off(a.sdq, b, tok, h) + ch * 8) =
        *reinterpret_cast<const uint4*>(region + tile_off(row, ch));
  }
}

}  // namespace

int launch_bwd_dq_spill_bf16(const KArgs& a, hipStream_t st) {
  const int NG = a.N / a.G;
  const int T = a.G / 128;
  const int n_rest = a.B * a.c_count * NG;
  const int il = interleave_for(T, 32);   // 32 CUs per XCD, one workgroup each
  const int blocks = 8 * T * pad_to(a.r * ((n_rest + 7) / 8), il);
  hipLaunchKernelGGL(bwd_dq_spill_kernel, dim3(blocks), dim3(256), 0, st, a, T, il, n_rest);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace s2
