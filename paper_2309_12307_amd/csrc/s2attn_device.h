// Shared between the host API and the kernels: the launch argument block and the
// shift/group index map of S2-Attn (LongLoRA Section 3.2, Algorithm 1).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s2 {

// Element strides of one tensor: batch, token, head (the head-dim axis is contiguous).
struct TStride {
  long long b, t, h;
};

struct KArgs {
  const void* q; const void* k; const void* v;
  void* o; float* lse;                       // forward outputs / backward inputs
  const void* dout;
  void* dq; void* dk; void* dv;
  float* delta;                              // (B,H,N) fp32
  float* lse2;                               // (B,H,N) fp32: lse * log2(e), written by the pre-pass
  float* dkv_partial;                        // fp32 [2 tensors][2 classes][B,N,Hkv,D] or null
  void* ds_spill;                            // bf16 dS tiles handed from the dK/dV kernel to the dQ kernel, or null
  int c_begin, c_count;                      // kv heads [c_begin, c_begin + c_count) of this launch (spill path)
  TStride sq, sk, sv, sdq, sdk, sdv;         // q, k, v and their gradients may be strided views
  TStride so;                                // o and dout: contiguous (B,N,H,D)
  int B, N, H, Hkv, D, G;
  int r;                                     // H / Hkv
  int shift;                                 // tokens, 0 <= shift < G
  int shifted_from;                          // heads >= shifted_from use the shifted partition
  int split;                                 // Variant 2: rows [0,split) | [split,G) of the wrap group; G = off
  int mixed;                                 // some kv head serves both head classes
  int ragged;                                // bf16 path: G % 128 != 0, shift % 64 != 0 or a Variant 2 split that
                                             // is not a multiple of 128 (partial tiles, wrap point inside a tile)
  float scale;                               // softmax scale
  float scale_log2;                          // scale * log2(e)
};

// Rolled position p of a head with shift s holds token (p + s) mod N
// (roll(x, -s) in Algorithm 1's first key line; both p and s are < N).
__device__ __forceinline__ int token_of(int p, int s, int N) {
  int t = p + s;
  return t >= N ? t - N : t;
}

// Element offset of row (batch b, token t, head h) of a tensor.
__device__ __forceinline__ size_t row_off(const TStride& s, int b, int t, int h) {
  return (size_t)((long long)b * s.b + (long long)t * s.t + (long long)h * s.h);
}

// A causal run: `len` consecutive rolled positions starting at `p0` inside which row i
// sees rows 0 .. i.  Normally a whole group (p0 = g * G, len = G); under Variant 2
// (Appendix B.3) the wrap-around group of a shifted head is two runs, [0, split) and
// [split, G) of the group.
struct Run {
  int p0, len;
};

// Token of row i of a run, with rows past its end (padding of a partial tile) clamped to
// the last row so that every load stays inside the tensor.
__device__ __forceinline__ int run_token(const KArgs& a, const Run& run, int i, int s) {
  return token_of(run.p0 + min(i, run.len - 1), s, a.N);
}

__device__ __forceinline__ int shift_of_head(const KArgs& a, int h) {
  return h >= a.shifted_from ? a.shift : 0;
}

// First visible key index for query row i of group g (0 except under Variant 2
// in the wrap-around group of a shifted head, Appendix B.3).
__device__ __forceinline__ int split_of_group(const KArgs& a, int g, int s) {
  return (s > 0 && g == a.N / a.G - 1) ? a.split : a.G;   // a.split == G means "no split"
}

// Block slot of one XCD -> (y, rank): y numbers the independent tile sequences of the launch
// (one per batch, head, group ...), rank orders the T tiles of a sequence from heaviest (0)
// to lightest.  `il` sequences are walked together, heaviest tiles of all of them first:
// when a sequence has fewer tiles than the XCD has workgroup slots, several sequences are
// resident anyway, and this order hands every slot about the same total work (a plain
// sequence-by-sequence order leaves the slots that drew heavy tiles running at the end).
__device__ __forceinline__ void decode_slot(int slot, int T, int il, int& y, int& rank) {
  const int span = T * il;
  const int chunk = __builtin_amdgcn_readfirstlane(slot / span);
  const int within = slot - chunk * span;
  rank = __builtin_amdgcn_readfirstlane(within / il);
  y = chunk * il + (within - rank * il);
}

// ---- dS hand-over between the two backward kernels (tile-aligned shapes only).
// The dK/dV kernel stores dS = P * (dP - delta) of every (64 queries x 128 keys) tile it
// visits as one 16 KB blob, exactly as its waves hold it: [key block kb 0..3][operand f 0..3]
// [lane 0..63][8 bf16], where lane = 32 g + (key % 32) of the wave that owns keys
// 32 kb .. 32 kb + 31, and element e of the lane's f-th packed operand is query
// 32 (f / 2) + 16 (f % 2) + 8 (e / 4) + 4 g + (e % 4) of the tile.  Every store instruction
// of a wave therefore writes 1 KB of consecutive bytes.  Seen as a matrix with one row per
// key and the 64 queries along the columns in the order (f, g, e), the column index within
// every 16 queries is the query index with bits 2 and 3 exchanged.  The dQ kernel reads the
// blobs back instead of recomputing S and dP.
// Blobs of one (batch, query head, group) are ordered by key tile jt (128 keys), then by
// query tile it = 0, 1, ... counted from the diagonal (query rows 128 jt + 64 it ...); a key
// tile has 2 (T - jt) query tiles when the group has T key tiles.
constexpr int kDsBlobBytes = 64 * 128 * 2;
__host__ __device__ inline long long ds_blobs_per_group(int T) { return (long long)T * (T + 1); }
__host__ __device__ inline long long ds_blob_index(int T, int jt, int it) {
  return (long long)jt * (2 * T - jt + 1) + it;
}
// Query row (within its 16) of column `col` (within its 16) of a blob, and back: bits 2 and 3
// exchanged.
__host__ __device__ inline int ds_col_query(int col) {
  return (col & ~12) | ((col & 4) << 1) | ((col & 8) >> 1);
}

// Kernels built for partial tiles treat Variant 2 by running the two halves of the
// wrap-around group as causal runs of their own: tile index `t` of the group (tiles of
// `tile` rows, first run's tiles first) -> the run and the tile index inside it.  Returns
// false when the group has no such tile (the grid is sized for the worst case).
__device__ __forceinline__ bool run_of_tile(const KArgs& a, int g, int s, int tile, int& t, Run& run) {
  run.p0 = g * a.G;
  run.len = a.G;
  const int split = split_of_group(a, g, s);
  if (split < a.G) {
    const int t_first = (split + tile - 1) / tile;
    if (t < t_first) {
      run.len = split;
    } else {
      t -= t_first;
      run.p0 += split;
      run.len = a.G - split;
    }
  }
  return t * tile < run.len;
}

// Tiles of `tile` rows that a group needs at most under run_of_tile.
inline int ragged_tiles(const KArgs& a, int tile) {
  const int whole = (a.G + tile - 1) / tile;
  if (a.split >= a.G) return whole;
  const int two = (a.split + tile - 1) / tile + (a.G - a.split + tile - 1) / tile;
  return two > whole ? two : whole;
}

}  // namespace s2
