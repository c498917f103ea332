// Host side of the C ABI declared in include/s2attn.h: argument checks, workspace
// layout, translation of the public parameter block into the kernels' argument
// block, and kernel launches.  Nothing here allocates device memory.
#include "s2attn.h"

#include <atomic>
#include <algorithm>
#include <cmath>
#include <cstring>

#include "s2attn_device.h"
#include "s2attn_launch.h"

namespace {

constexpr size_t kAlign = 256;

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// First head that uses the shifted partition under a rule (Algorithm 1 shifts the
// second chunk of chunk(2, head axis)).
int shifted_from(int rule, int H, int shift, int heads_total = 0, int head_offset = 0) {
  if (shift == 0) return H;
  switch (rule) {
    case S2ATTN_SHIFT_SECOND_HALF:
      // head-sharded: local index of the layer's head heads_total / 2, clamped to this shard
      if (heads_total > 0) return std::min(std::max(heads_total / 2 - head_offset, 0), H);
      return H / 2;
    case S2ATTN_SHIFT_NONE: return H;
    default: return 0;
  }
}

int shifted_from(const s2attn_params* p, int shift) {
  return shifted_from(p->shift_rule, p->H, shift, p->heads_total, p->head_offset);
}

int resolved_shift(const s2attn_params* p) { return p->shift < 0 ? p->G / 2 : p->shift; }

// A kv head is "mixed" when its query heads fall on both sides of shifted_from.
bool kv_heads_mixed(int H, int Hkv, int from) {
  const int r = H / Hkv;
  return from > 0 && from < H && (from % r) != 0;
}

size_t delta_bytes(int B, int N, int H) { return round_up((size_t)B * H * N * sizeof(float), kAlign); }

size_t workspace_bytes_for(int B, int N, int H, int Hkv, int D, bool mixed) {
  size_t w = 2 * delta_bytes(B, N, H);   // delta and lse * log2(e)
  if (mixed) w += round_up((size_t)4 * B * N * Hkv * D * sizeof(float), kAlign);
  return w;
}

// ---- stored-dS backward (tile-aligned bf16 shapes): the dK/dV kernel hands dS to the dQ
// kernel through the workspace, one kv head's query heads after the other.
constexpr size_t kDsSpillCap = (size_t)16 << 30;   // what the workspace queries ask for at most

// Shapes the role-split dK/dV kernel (and so the stored-dS path) accepts.
bool stored_ds_applies(const s2attn_params* p, int shift, int from) {
  if (p->dtype != S2ATTN_BF16 || p->D != 128) return false;
  if (p->G % 128 != 0 || shift % 64 != 0) return false;
  if (p->wrap_variant == S2ATTN_WRAP_SPLIT && shift > 0 && (p->G - shift) % 128 != 0) return false;
  return !kv_heads_mixed(p->H, p->Hkv, from);
}

// dS bytes of all query heads of one kv head: 2 bytes per (query, key) pair of the tiles at or
// below the diagonal.
size_t ds_bytes_per_kv_head(const s2attn_params* p) {
  const size_t T = (size_t)p->G / 128;
  return (size_t)p->B * (p->H / p->Hkv) * (p->N / p->G) * T * (T + 1) * s2::kDsBlobBytes;
}

// kv heads whose dS fits into `avail` bytes at a time (0: none).
int ds_heads_per_pass(const s2attn_params* p, size_t avail) {
  const size_t per_head = ds_bytes_per_kv_head(p);
  const size_t n = avail / per_head;
  return (int)std::min<size_t>(n, (size_t)p->Hkv);
}

// Workspace a parameter block asks for: the row terms (and partial sums), plus, when the block
// asks for the stored-dS backward, room for the dS of as many kv heads as fit under the cap (at
// least one).
size_t workspace_bytes_wanted(const s2attn_params* p) {
  const int shift = resolved_shift(p);
  const int from = shifted_from(p, shift);
  size_t w = workspace_bytes_for(p->B, p->N, p->H, p->Hkv, p->D, kv_heads_mixed(p->H, p->Hkv, from));
  if (p->bwd_algo == S2ATTN_BWD_STORED_DS && stored_ds_applies(p, shift, from)) {
    const size_t per_head = ds_bytes_per_kv_head(p);
    const size_t heads = std::max<size_t>(1, std::min<size_t>((size_t)p->Hkv, kDsSpillCap / per_head));
    w += heads * per_head;
  }
  return w;
}

bool strides_ok(const long long (&st)[3], int B, int heads, int D, int align) {
  if (st[0] == 0 && st[1] == 0 && st[2] == 0) return true;
  for (long long x : st)
    if (x < 0 || x % align != 0) return false;
  if (st[2] < D && heads > 1) return false;
  if (st[1] < D) return false;
  if (st[1] >= (1LL << 26)) return false;   // kernels keep (row within a tile) * token stride in 32 bits
  if (st[0] < D && B > 1) return false;
  return true;
}

// Output tensors must not alias themselves: ordering the three strided axes by stride, each
// stride has to cover the whole extent of the axes below it (the head-dim axis, D contiguous
// elements, is the innermost).
bool rows_disjoint(const long long (&st)[3], int B, int N, int heads, int D) {
  if (st[0] == 0 && st[1] == 0 && st[2] == 0) return true;
  struct Axis { long long stride; long long extent; };
  Axis ax[3] = {{st[0], B}, {st[1], N}, {st[2], heads}};
  std::sort(ax, ax + 3, [](const Axis& x, const Axis& y) { return x.stride < y.stride; });
  long long span = D;   // elements covered by everything below the current axis
  for (const Axis& x : ax) {
    if (x.extent <= 1) continue;
    if (x.stride < span) return false;
    span = x.stride * (x.extent - 1) + span;
  }
  return true;
}

int check_common(const s2attn_params* p, int backward) {
  if (!p) return S2ATTN_ERR_NULL;
  if (p->dtype != S2ATTN_BF16 && p->dtype != S2ATTN_F32) return S2ATTN_ERR_DTYPE;
  if (p->shift_rule < S2ATTN_SHIFT_SECOND_HALF || p->shift_rule > S2ATTN_SHIFT_ALL) return S2ATTN_ERR_DTYPE;
  if (p->wrap_variant != S2ATTN_WRAP_JOINT && p->wrap_variant != S2ATTN_WRAP_SPLIT) return S2ATTN_ERR_DTYPE;
  if (p->bwd_algo < S2ATTN_BWD_AUTO || p->bwd_algo > S2ATTN_BWD_STORED_DS) return S2ATTN_ERR_DTYPE;
  if (p->B <= 0 || p->N <= 0 || p->H <= 0 || p->Hkv <= 0 || p->D <= 0 || p->G <= 0) return S2ATTN_ERR_DIM;
  if (p->N % p->G != 0 || p->G % 2 != 0) return S2ATTN_ERR_GROUP;
  const int shift = resolved_shift(p);
  if (shift < 0 || shift >= p->G) return S2ATTN_ERR_GROUP;
  if (p->H % p->Hkv != 0) return S2ATTN_ERR_HEADS;
  if (p->heads_total == 0) {
    if (p->H % 2 != 0 || p->head_offset != 0) return S2ATTN_ERR_HEADS;
  } else {
    if (p->heads_total < 0 || p->heads_total % 2 != 0 || p->head_offset < 0 ||
        (long long)p->head_offset + p->H > p->heads_total || p->head_offset % (p->H / p->Hkv) != 0)
      return S2ATTN_ERR_HEADS;
  }
  if (p->D != 64 && p->D != 128) return S2ATTN_ERR_HEADDIM;
  // grid z carries batch * heads (* 2 classes); element offsets are 64-bit
  if ((long long)p->B * p->H * 2 > 65535 || (long long)p->N / p->G > 65535) return S2ATTN_ERR_TOO_LARGE;
  if ((double)p->B * p->N * p->H * p->D > 9.0e18 / 4) return S2ATTN_ERR_TOO_LARGE;

  const int align = p->dtype == S2ATTN_F32 ? 4 : 8;
  if (!strides_ok(p->q_strides, p->B, p->H, p->D, align) || !strides_ok(p->k_strides, p->B, p->Hkv, p->D, align) ||
      !strides_ok(p->v_strides, p->B, p->Hkv, p->D, align))
    return S2ATTN_ERR_STRIDE;
  if (backward && (!strides_ok(p->dq_strides, p->B, p->H, p->D, align) ||
                   !strides_ok(p->dk_strides, p->B, p->Hkv, p->D, align) ||
                   !strides_ok(p->dv_strides, p->B, p->Hkv, p->D, align)))
    return S2ATTN_ERR_STRIDE;
  if (backward && (!rows_disjoint(p->dq_strides, p->B, p->N, p->H, p->D) ||
                   !rows_disjoint(p->dk_strides, p->B, p->N, p->Hkv, p->D) ||
                   !rows_disjoint(p->dv_strides, p->B, p->N, p->Hkv, p->D)))
    return S2ATTN_ERR_STRIDE;
  const void* need_fwd[] = {p->q, p->k, p->v, p->o, p->lse};
  for (const void* x : need_fwd) {
    if (!x) return S2ATTN_ERR_NULL;
    if (!aligned16(x)) return S2ATTN_ERR_ALIGN;
  }
  if (backward) {
    const void* need_bwd[] = {p->dout, p->dq, p->dk, p->dv};
    for (const void* x : need_bwd) {
      if (!x) return S2ATTN_ERR_NULL;
      if (!aligned16(x)) return S2ATTN_ERR_ALIGN;
    }
    const int from = shifted_from(p, shift);
    const bool mixed = kv_heads_mixed(p->H, p->Hkv, from);
    const size_t need = workspace_bytes_for(p->B, p->N, p->H, p->Hkv, p->D, mixed);
    if (!p->workspace || p->workspace_bytes < need) return S2ATTN_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(p->workspace) & (kAlign - 1)) != 0) return S2ATTN_ERR_ALIGN;
    if (p->bwd_algo == S2ATTN_BWD_STORED_DS) {
      if (!stored_ds_applies(p, shift, from)) return S2ATTN_ERR_ALGO;
      if (ds_heads_per_pass(p, p->workspace_bytes - need) == 0) return S2ATTN_ERR_WORKSPACE;
    }
  }
  return S2ATTN_OK;
}

// The kernels use gfx950-only instructions; refuse any other device.  The answer
// per device ordinal is cached (0 unknown, 1 yes, 2 no).
int check_device() {
  static std::atomic<int> cache[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return S2ATTN_ERR_DEVICE;
  int state = (dev >= 0 && dev < 64) ? cache[dev].load(std::memory_order_relaxed) : 0;
  if (state == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return S2ATTN_ERR_DEVICE;
    state = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 2;
    if (dev >= 0 && dev < 64) cache[dev].store(state, std::memory_order_relaxed);
  }
  return state == 1 ? S2ATTN_OK : S2ATTN_ERR_DEVICE;
}

// Strides of a tensor with `heads` heads: the caller's, or contiguous (B, N, heads, D) when all zero.
s2::TStride resolve_strides(const long long (&st)[3], int N, int heads, int D) {
  s2::TStride r;
  if (st[0] == 0 && st[1] == 0 && st[2] == 0) {
    r.b = (long long)N * heads * D; r.t = (long long)heads * D; r.h = D;
  } else {
    r.b = st[0]; r.t = st[1]; r.h = st[2];
  }
  return r;
}

s2::KArgs make_kargs(const s2attn_params* p) {
  s2::KArgs a;
  std::memset(&a, 0, sizeof(a));
  a.q = p->q; a.k = p->k; a.v = p->v; a.o = p->o; a.lse = p->lse;
  a.dout = p->dout; a.dq = p->dq; a.dk = p->dk; a.dv = p->dv;
  a.B = p->B; a.N = p->N; a.H = p->H; a.Hkv = p->Hkv; a.D = p->D; a.G = p->G;
  a.r = p->H / p->Hkv;
  a.sq = resolve_strides(p->q_strides, p->N, p->H, p->D);
  a.sk = resolve_strides(p->k_strides, p->N, p->Hkv, p->D);
  a.sv = resolve_strides(p->v_strides, p->N, p->Hkv, p->D);
  a.sdq = resolve_strides(p->dq_strides, p->N, p->H, p->D);
  a.sdk = resolve_strides(p->dk_strides, p->N, p->Hkv, p->D);
  a.sdv = resolve_strides(p->dv_strides, p->N, p->Hkv, p->D);
  const long long zero3[3] = {0, 0, 0};
  a.so = resolve_strides(zero3, p->N, p->H, p->D);
  a.shift = resolved_shift(p);
  a.shifted_from = shifted_from(p, a.shift);
  a.split = (p->wrap_variant == S2ATTN_WRAP_SPLIT && a.shift > 0) ? p->G - a.shift : p->G;
  a.mixed = kv_heads_mixed(p->H, p->Hkv, a.shifted_from) ? 1 : 0;
  // the kernels built for partial tiles also take rows narrower than the 128-element tile (D = 64)
  a.ragged = (p->dtype == S2ATTN_BF16 && (p->D != 128 || p->G % 128 != 0 || a.shift % 64 != 0 ||
                                          (a.split < p->G && a.split % 128 != 0))) ? 1 : 0;
  a.c_begin = 0;
  a.c_count = p->Hkv;
  a.scale = p->scale > 0.f ? p->scale : 1.0f / std::sqrt((float)p->D);
  a.scale_log2 = a.scale * 1.4426950408889634f;
  return a;
}

s2attn_params basic_params(const void* q, const void* k, const void* v, void* o, float* lse,
                           int B, int N, int H, int Hkv, int D, int G, int dtype) {
  s2attn_params p;
  std::memset(&p, 0, sizeof(p));
  p.q = q; p.k = k; p.v = v; p.o = o; p.lse = lse;
  p.B = B; p.N = N; p.H = H; p.Hkv = Hkv; p.D = D; p.G = G;
  p.dtype = dtype;
  p.shift = -1;
  p.shift_rule = S2ATTN_SHIFT_SECOND_HALF;
  p.wrap_variant = S2ATTN_WRAP_JOINT;
  p.scale = 0.f;
  return p;
}

}  // namespace

extern "C" {

int s2attn_check_args(const s2attn_params* p, int backward) { return check_common(p, backward); }

size_t s2attn_bwd_workspace_bytes(int B, int N, int H, int Hkv, int D, int G, int dtype) {
  // the published defaults: shift G/2 on the second half of the heads, one causal wrap group
  s2attn_params p = basic_params(nullptr, nullptr, nullptr, nullptr, nullptr, B, N, H, Hkv, D, G, dtype);
  return s2attn_bwd_workspace_bytes_ex(&p);
}

size_t s2attn_bwd_workspace_bytes_ex(const s2attn_params* p) {
  if (!p || p->B <= 0 || p->N <= 0 || p->H <= 0 || p->Hkv <= 0 || p->D <= 0 || p->G <= 0 || p->H % p->Hkv != 0 ||
      p->N % p->G != 0)
    return 0;
  return workspace_bytes_wanted(p);
}

int s2attn_fwd_ex(const s2attn_params* p, void* stream) {
  int rc = check_common(p, 0);
  if (rc != S2ATTN_OK) return rc;
  rc = check_device();
  if (rc != S2ATTN_OK) return rc;
  s2::KArgs a = make_kargs(p);
  hipStream_t st = static_cast<hipStream_t>(stream);
  rc = p->dtype == S2ATTN_F32 ? s2::launch_fwd_f32(a, st) : s2::launch_fwd_bf16(a, st);
  return rc == 0 ? S2ATTN_OK : S2ATTN_ERR_LAUNCH;
}

static int run_bwd(const s2attn_params* p, void* stream, void* const* events) {
  int rc = check_common(p, 1);
  if (rc != S2ATTN_OK) return rc;
  rc = check_device();
  if (rc != S2ATTN_OK) return rc;
  s2::KArgs a = make_kargs(p);
  a.delta = static_cast<float*>(p->workspace);
  a.lse2 = reinterpret_cast<float*>(static_cast<char*>(p->workspace) + delta_bytes(p->B, p->N, p->H));
  if (a.mixed)
    a.dkv_partial = reinterpret_cast<float*>(static_cast<char*>(p->workspace) + 2 * delta_bytes(p->B, p->N, p->H));
  hipStream_t st = static_cast<hipStream_t>(stream);
  auto mark = [&](int i) {
    if (events && events[i]) (void)hipEventRecord(static_cast<hipEvent_t>(events[i]), st);
  };
  // stored-dS backward: only on request (check_common has made sure that the shape allows it
  // and that the workspace has room for the dS of at least one kv head beyond the row terms)
  const size_t basic = workspace_bytes_for(p->B, p->N, p->H, p->Hkv, p->D, a.mixed != 0);
  int ds_heads = 0;
  if (p->bwd_algo == S2ATTN_BWD_STORED_DS) ds_heads = ds_heads_per_pass(p, p->workspace_bytes - basic);
  mark(0);
  if (s2::launch_delta(a, p->dtype, st) != 0) return S2ATTN_ERR_LAUNCH;
  mark(1);
  if (ds_heads > 0) {
    // kv heads in passes of ds_heads: dK/dV kernel (stores dS), then dQ from the stored dS
    a.ds_spill = static_cast<char*>(p->workspace) + basic;
    for (int c0 = 0; c0 < p->Hkv; c0 += ds_heads) {
      a.c_begin = c0;
      a.c_count = std::min(ds_heads, p->Hkv - c0);
      if (s2::launch_bwd_dkdv_split_bf16(a, st) != 0) return S2ATTN_ERR_LAUNCH;
      if (c0 + ds_heads >= p->Hkv) mark(2);
      if (s2::launch_bwd_dq_spill_bf16(a, st) != 0) return S2ATTN_ERR_LAUNCH;
    }
    mark(3);
    return S2ATTN_OK;
  }
  rc = p->dtype == S2ATTN_F32 ? s2::launch_bwd_dkdv_f32(a, st) : s2::launch_bwd_dkdv_bf16(a, st);
  if (rc != 0) return S2ATTN_ERR_LAUNCH;
  mark(2);
  rc = p->dtype == S2ATTN_F32 ? s2::launch_bwd_dq_f32(a, st) : s2::launch_bwd_dq_bf16(a, st);
  if (rc != 0) return S2ATTN_ERR_LAUNCH;
  if (a.mixed && s2::launch_combine_partials(a, p->dtype, st) != 0) return S2ATTN_ERR_LAUNCH;
  mark(3);
  return S2ATTN_OK;
}

int s2attn_bwd_ex(const s2attn_params* p, void* stream) { return run_bwd(p, stream, nullptr); }

// ---- backward without a caller workspace: the row terms (and, for a kv head that serves both
// head classes, the fp32 partial sums) live in a device array that is part of the library's
// code object.  Every GPU the library runs on holds its own copy at its own address, so the
// address is looked up once per device, with that device current, and cached.
namespace {
static __device__ __align__(256) unsigned char scratch[S2ATTN_STATIC_SCRATCH_BYTES];
std::atomic<void*> scratch_ptr[64];

int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return S2ATTN_ERR_DEVICE;
  void* ptr = scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return S2ATTN_ERR_DEVICE;
    scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return S2ATTN_OK;
}
}  // namespace

int s2attn_bwd_ex_static(const s2attn_params* p, void* stream) {
  if (!p) return S2ATTN_ERR_NULL;
  s2attn_params local = *p;
  local.bwd_algo = S2ATTN_BWD_RECOMPUTE;   // the stored-dS backward needs gigabytes of workspace
  // size check first: pure host arithmetic, nothing is looked up or launched for a problem
  // that does not fit
  const size_t need = s2attn_bwd_workspace_bytes_ex(&local);
  if (need > S2ATTN_STATIC_SCRATCH_BYTES) return S2ATTN_ERR_SCRATCH;
  // the remaining argument errors do not depend on the workspace address
  local.workspace = reinterpret_cast<void*>(static_cast<uintptr_t>(kAlign));
  local.workspace_bytes = S2ATTN_STATIC_SCRATCH_BYTES;
  int rc = check_common(&local, 1);
  if (rc != S2ATTN_OK) return rc;
  rc = check_device();
  if (rc != S2ATTN_OK) return rc;
  void* ptr = nullptr;
  rc = static_scratch(&ptr);
  if (rc != S2ATTN_OK) return rc;
  local.workspace = ptr;
  return run_bwd(&local, stream, nullptr);
}

int s2attn_bwd_ex_marked(const s2attn_params* p, void* stream, void* const* events) {
  return run_bwd(p, stream, events);
}

int s2attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
               int B, int N, int H, int Hkv, int D, int G, void* stream) {
  s2attn_params p = basic_params(q, k, v, o, lse, B, N, H, Hkv, D, G, S2ATTN_BF16);
  return s2attn_fwd_ex(&p, stream);
}

int s2attn_fwd_f32(const float* q, const float* k, const float* v, float* o, float* lse,
                   int B, int N, int H, int Hkv, int D, int G, void* stream) {
  s2attn_params p = basic_params(q, k, v, o, lse, B, N, H, Hkv, D, G, S2ATTN_F32);
  return s2attn_fwd_ex(&p, stream);
}

int s2attn_bwd(const void* q, const void* k, const void* v, const void* o,
               const void* dout, const float* lse, void* dq, void* dk, void* dv,
               void* workspace, size_t workspace_bytes,
               int B, int N, int H, int Hkv, int D, int G, void* stream) {
  s2attn_params p = basic_params(q, k, v, const_cast<void*>(o), const_cast<float*>(lse),
                                 B, N, H, Hkv, D, G, S2ATTN_BF16);
  p.dout = dout; p.dq = dq; p.dk = dk; p.dv = dv;
  p.workspace = workspace; p.workspace_bytes = workspace_bytes;
  return s2attn_bwd_ex(&p, stream);
}

int s2attn_bwd_f32(const float* q, const float* k, const float* v, const float* o,
                   const float* dout, const float* lse, float* dq, float* dk, float* dv,
                   void* workspace, size_t workspace_bytes,
                   int B, int N, int H, int Hkv, int D, int G, void* stream) {
  s2attn_params p = basic_params(q, k, v, const_cast<float*>(o), const_cast<float*>(lse),
                                 B, N, H, Hkv, D, G, S2ATTN_F32);
  p.dout = dout; p.dq = dq; p.dk = dk; p.dv = dv;
  p.workspace = workspace; p.workspace_bytes = workspace_bytes;
  return s2attn_bwd_ex(&p, stream);
}

const char* s2attn_strerror(int code) {
  switch (code) {
    case S2ATTN_OK: return "ok";
    case S2ATTN_ERR_NULL: return "a required pointer is NULL";
    case S2ATTN_ERR_ALIGN: return "a tensor pointer is not 16-byte aligned (workspace: 256-byte)";
    case S2ATTN_ERR_DIM: return "B, N, H, Hkv, D and G must be positive";
    case S2ATTN_ERR_GROUP: return "need N % G == 0, G even and 0 <= shift < G";
    case S2ATTN_ERR_HEADS: return "need H even and H % Hkv == 0";
    case S2ATTN_ERR_HEADDIM: return "unsupported head dimension (64 or 128)";
    case S2ATTN_ERR_WORKSPACE: return "backward workspace missing or smaller than s2attn_bwd_workspace_bytes";
    case S2ATTN_ERR_DTYPE: return "unknown dtype, shift rule or wrap variant";
    case S2ATTN_ERR_DEVICE: return "current device is not gfx950 (MI355X)";
    case S2ATTN_ERR_LAUNCH: return "HIP kernel launch failed";
    case S2ATTN_ERR_TOO_LARGE: return "problem too large for the launch grid or index arithmetic";
    case S2ATTN_ERR_STRIDE: return "a stride is negative, misaligned or smaller than the extent it spans";
    case S2ATTN_ERR_ALGO: return "S2ATTN_BWD_STORED_DS needs bf16, G a multiple of 128, shift (and a Variant 2 split) of 64 (128), and no kv head serving both head classes";
    case S2ATTN_ERR_SCRATCH: return "the backward needs more scratch than the library's static 16 MiB: call s2attn_bwd_ex with a workspace";
    default: return "unknown s2attn error code";
  }
}

double s2attn_effective_flops(int B, int N, int H, int D, int G, int pass) {
  const double pairs = (double)B * H * N * (G + 1) / 2.0;
  const double per_pair = pass == 0 ? 4.0 : (pass == 1 ? 10.0 : 14.0);
  return pairs * D * per_pair;
}

}  // extern "C"
