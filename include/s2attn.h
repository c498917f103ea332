/* s2attn.h -- C ABI of the MI355X (gfx950) shifted sparse attention library.
 *
 * The operation is S2-Attn of LongLoRA (arXiv 2309.12307), Section 3.2 and
 * Algorithm 1: the N tokens are cut into N/G groups of G tokens; for the second
 * contiguous half of the query heads the partition is shifted by G/2 tokens with
 * wrap-around (token t sits at rolled position (t - G/2) mod N); softmax
 * attention (Equation 1, with the 1/sqrt(D) scale and the causal mask of a
 * standard decoder self-attention, both in the rolled in-group index) runs inside
 * every group; outputs land at their original token rows.  No rolled copy of any
 * tensor is made: the roll only changes which rows a tile reads and writes.
 *
 * Conventions common to every call
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or keeps them.  `stream` is a hipStream_t passed as
 *     void* (NULL = the default stream).  Calls only enqueue work and return.
 *   - Layouts are contiguous row-major: q, o, dout, dq are (B, N, H, D);
 *     k, v, dk, dv are (B, N, Hkv, D); lse is (B, H, N) fp32 and holds the natural
 *     log of the sum of exp of the scaled, masked scores of each ORIGINAL token.
 *   - Grouped-query attention: query head h reads kv head h / (H/Hkv); whether a
 *     head is shifted is a property of the query head; dk, dv sum over the query
 *     heads that share a kv head.
 *   - Return value: 0 (S2ATTN_OK) or a negative S2ATTN_ERR_* code.  Argument errors
 *     are found before anything is launched.  S2ATTN_ERR_LAUNCH means HIP refused a
 *     kernel launch: the backward enqueues several kernels, so earlier ones of the
 *     same call may already be on the stream and the outputs are then undefined.
 *     The library has no mutable global state; calls are re-entrant and may be
 *     issued from several host threads.
 *   - bf16 calls take any even G and any shift; G a multiple of 128 with the shift
 *     (and, under Variant 2, G - shift) a multiple of 64 (128) runs the faster
 *     tile-aligned kernels.
 *   - Tensor pointers must be 16-byte aligned.
 */
#ifndef S2ATTN_H
#define S2ATTN_H

#include <stddef.h>

#if defined(__GNUC__)
#define S2ATTN_API __attribute__((visibility("default")))
#else
#define S2ATTN_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

enum {
  S2ATTN_OK = 0,
  S2ATTN_ERR_NULL = -1,        /* a required pointer is NULL */
  S2ATTN_ERR_ALIGN = -2,       /* a tensor pointer is not 16-byte aligned */
  S2ATTN_ERR_DIM = -3,         /* B, N, H, Hkv, D or G is not positive */
  S2ATTN_ERR_GROUP = -4,       /* N % G != 0, or G odd, or shift outside [0, G) */
  S2ATTN_ERR_HEADS = -5,       /* H odd (half of the heads shift), H % Hkv != 0, or inconsistent head sharding */
  S2ATTN_ERR_HEADDIM = -6,     /* D not supported: D must be 64 or 128 */
  /* -7 is unused (it was a tile-alignment error that no longer exists) */
  S2ATTN_ERR_WORKSPACE = -8,   /* backward workspace missing or too small */
  S2ATTN_ERR_DTYPE = -9,       /* unknown dtype / rule / variant value */
  S2ATTN_ERR_DEVICE = -10,     /* current device is not gfx950 */
  S2ATTN_ERR_LAUNCH = -11,     /* HIP reported a launch error */
  S2ATTN_ERR_TOO_LARGE = -12,  /* tensor too large for the index arithmetic, or over a fixed limit */
  S2ATTN_ERR_STRIDE = -13,     /* a stride is negative, misaligned or smaller than the extent it spans */
  S2ATTN_ERR_SCRATCH = -14,    /* s2attn_bwd_ex_static: the problem needs more than S2ATTN_STATIC_SCRATCH_BYTES */
  S2ATTN_ERR_ALGO = -15        /* S2ATTN_BWD_STORED_DS asked for a shape it does not cover */
};

enum { S2ATTN_BF16 = 0, S2ATTN_F32 = 1 };

/* Which query heads use the shifted partition (Section 3.2; the attention-pattern
 * ablation of Section 4.3 uses the other two). */
enum {
  S2ATTN_SHIFT_SECOND_HALF = 0, /* heads [H/2, H): the method as published */
  S2ATTN_SHIFT_NONE = 1,        /* no head shifts ("pattern 1" only; with G == N: full causal attention) */
  S2ATTN_SHIFT_ALL = 2          /* every head shifts ("pattern 2" only) */
};

/* Treatment of the wrap-around group of shifted heads (last `shift` tokens
 * followed by the first `shift` tokens; Appendix B.3). */
enum {
  S2ATTN_WRAP_JOINT = 0,  /* one causal group: the paper's default method */
  S2ATTN_WRAP_SPLIT = 2   /* "Variant 2": the two halves are separate groups */
};

/* How the backward's dQ kernel obtains dS = P * (dP - delta) (the gradient formulas are the same;
 * the paper leaves the backward to autograd).  Measured on MI355X at the 7B-shaped N = 32768
 * layer the two take the same time to within 2 %, so the default is the one without the large
 * workspace. */
enum {
  S2ATTN_BWD_AUTO = 0,       /* the library's choice: currently S2ATTN_BWD_RECOMPUTE */
  S2ATTN_BWD_RECOMPUTE = 1,  /* the dQ kernel recomputes S and dP: workspace of a few MB, 18 D flops
                                executed per (query, key) pair for forward + backward */
  S2ATTN_BWD_STORED_DS = 2   /* the dK/dV kernel stores dS (bf16, 2 bytes per pair) in the workspace and
                                the dQ kernel reads it back: 14 D flops per pair, 4 bytes of HBM traffic
                                per pair.  bf16, G % 128 == 0, shift % 64 == 0, (G - shift) % 128 == 0
                                under Variant 2, no kv head serving shifted and unshifted query heads;
                                otherwise S2ATTN_ERR_ALGO.  The workspace must hold the dS of at least
                                one kv head beyond the row terms; kv heads then run in passes */
};

typedef struct s2attn_params {
  /* forward: q, k, v in; o, lse out.  backward: q, k, v, o, dout, lse in; dq, dk, dv out. */
  const void* q;
  const void* k;
  const void* v;
  void* o;            /* written by forward, read by backward */
  float* lse;         /* written by forward, read by backward */
  const void* dout;   /* backward only */
  void* dq;           /* backward only, overwritten */
  void* dk;           /* backward only, overwritten */
  void* dv;           /* backward only, overwritten */
  void* workspace;    /* backward only: >= s2attn_bwd_workspace_bytes(...) bytes, 256-byte aligned */
  size_t workspace_bytes;
  int B, N, H, Hkv, D, G;
  int dtype;          /* S2ATTN_BF16 or S2ATTN_F32: element type of q,k,v,o,dout,dq,dk,dv */
  int shift;          /* tokens; negative = G/2 (the paper's value) */
  int shift_rule;     /* S2ATTN_SHIFT_* */
  int wrap_variant;   /* S2ATTN_WRAP_* */
  float scale;        /* softmax scale; <= 0 means 1/sqrt(D) */
  /* Optional element strides {batch, token, head} of q, k, v, dq, dk, dv (the head-dim
   * axis is always contiguous).  All three zero = contiguous.  Lets the three slices of a
   * packed (B, N, 3, H, D) projection (Algorithm 1's qkv) be passed without a split copy:
   * {N*3*H*D, 3*H*D, D} with pointers offset by 0, H*D and 2*H*D elements.  Every stride
   * must be a multiple of 8 elements (bf16) or 4 (fp32) and the token stride below 2^26
   * elements; o, dout, lse stay contiguous. */
  long long q_strides[3], k_strides[3], v_strides[3];
  long long dq_strides[3], dk_strides[3], dv_strides[3];
  /* Head-sharded use (one GPU holds heads [head_offset, head_offset + H) of a layer with
   * heads_total query heads): under S2ATTN_SHIFT_SECOND_HALF the shifted heads are those whose
   * layer-wide index is >= heads_total / 2.  heads_total == 0 (the default) means the call
   * sees the whole layer (heads_total = H, head_offset = 0).  heads_total must be even,
   * head_offset + H <= heads_total and head_offset a multiple of H / Hkv; H itself may then
   * be odd. */
  int heads_total;
  int head_offset;
  int bwd_algo;       /* S2ATTN_BWD_*; backward only */
} s2attn_params;

/* Pure host check of a parameter block (pointers, alignment, shapes, workspace
 * size when `backward` is non-zero).  Touches no GPU state. */
S2ATTN_API int s2attn_check_args(const s2attn_params* p, int backward);

/* Bytes of device workspace the backward needs, for the published defaults (shift G/2 on the
 * second half of the heads): the fp32 row term delta[b,h,t] = sum_d dout*o and a base-2 copy of
 * lse, plus fp32 partial dk/dv when a kv head serves both shifted and unshifted query heads
 * (odd Hkv). */
S2ATTN_API size_t s2attn_bwd_workspace_bytes(int B, int N, int H, int Hkv, int D, int G, int dtype);

/* Same for a parameter block (accounts for its shift rule and head sharding, which decide
 * whether a kv head serves both kinds of query heads, and for bwd_algo: S2ATTN_BWD_STORED_DS
 * adds room for dS, 2 bytes per in-group causal (query, key) pair of as many kv heads as fit
 * into 16 GiB, at least one); 0 if the shape fields are invalid. */
S2ATTN_API size_t s2attn_bwd_workspace_bytes_ex(const s2attn_params* p);

/* Forward of Algorithm 1, bf16 tensors, fp32 accumulation, default shift G/2 on
 * heads [H/2, H), scale 1/sqrt(D). */
S2ATTN_API int s2attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
               int B, int N, int H, int Hkv, int D, int G, void* stream);

/* Backward of the same map: recomputes P from lse (softmax-Jacobian form
 * dS = P * (dP - delta)); overwrites dq, dk, dv. */
S2ATTN_API int s2attn_bwd(const void* q, const void* k, const void* v, const void* o,
               const void* dout, const float* lse, void* dq, void* dk, void* dv,
               void* workspace, size_t workspace_bytes,
               int B, int N, int H, int Hkv, int D, int G, void* stream);

/* Same two calls with fp32 tensors and fp32 arithmetic throughout. */
S2ATTN_API int s2attn_fwd_f32(const float* q, const float* k, const float* v, float* o, float* lse,
                   int B, int N, int H, int Hkv, int D, int G, void* stream);
S2ATTN_API int s2attn_bwd_f32(const float* q, const float* k, const float* v, const float* o,
                   const float* dout, const float* lse, float* dq, float* dk, float* dv,
                   void* workspace, size_t workspace_bytes,
                   int B, int N, int H, int Hkv, int D, int G, void* stream);

/* General forms: dtype, shift amount, which heads shift (Section 4.3 ablation
 * patterns), wrap-group variant (Appendix B.3) and scale come from the block. */
S2ATTN_API int s2attn_fwd_ex(const s2attn_params* p, void* stream);
S2ATTN_API int s2attn_bwd_ex(const s2attn_params* p, void* stream);

/* For callers that cannot allocate device memory or carry a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): s2attn_bwd_ex with the
 * workspace replaced by a device array of S2ATTN_STATIC_SCRATCH_BYTES that is part of the
 * library image (each GPU holds its own copy until the process ends).  p->workspace and
 * p->workspace_bytes are ignored; everything else, results included, is as in s2attn_bwd_ex.
 * It always runs the recomputing backward (p->bwd_algo is ignored).
 * The call allocates nothing and frees nothing.  A problem whose
 * s2attn_bwd_workspace_bytes_ex (without stored dS) exceeds S2ATTN_STATIC_SCRATCH_BYTES
 * (for MHA and even Hkv: B * H * N > 2097152 rows) is refused with S2ATTN_ERR_SCRATCH before anything is launched.
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU
 * (different streams, several host threads) race on it and must be serialised by the caller;
 * nothing in it needs to start at zero, and a call leaves nothing behind that a later call
 * reads. */
#define S2ATTN_STATIC_SCRATCH_BYTES (16u << 20)
S2ATTN_API int s2attn_bwd_ex_static(const s2attn_params* p, void* stream);

/* Measurement aid: s2attn_bwd_ex that also records up to four caller-owned HIP events
 * (hipEvent_t passed as void*, entries may be NULL) on `stream`: events[0] before the
 * delta pre-pass, [1] after it, [2] after the dK/dV kernel, [3] after the dQ kernel
 * (and the partial-sum pass, when present).  Same semantics and errors otherwise. */
S2ATTN_API int s2attn_bwd_ex_marked(const s2attn_params* p, void* stream, void* const* events);

/* Static, never-freed message for a return code. */
S2ATTN_API const char* s2attn_strerror(int code);

/* Effective FLOPs of one layer counting only in-group causal (query, key) pairs
 * (Equation 1 restricted to the groups of Section 3.2): 4*D per pair forward,
 * 10*D per pair backward.  pass: 0 = forward, 1 = backward, 2 = both. */
S2ATTN_API double s2attn_effective_flops(int B, int N, int H, int D, int G, int pass);

#ifdef __cplusplus
}
#endif
#endif /* S2ATTN_H */
