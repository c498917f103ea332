// Internal launch entry points, one per kernel family.  Each returns 0 or -1
// (HIP launch error) and only enqueues work on the given stream.
#pragma once
#include "s2attn_device.h"

namespace s2 {

int launch_fwd_f32(const KArgs& a, hipStream_t st);
int launch_bwd_dkdv_f32(const KArgs& a, hipStream_t st);   // delta must be ready
int launch_bwd_dq_f32(const KArgs& a, hipStream_t st);

int launch_fwd_bf16(const KArgs& a, hipStream_t st);
int launch_bwd_dkdv_bf16(const KArgs& a, hipStream_t st);  // delta must be ready
int launch_bwd_dq_bf16(const KArgs& a, hipStream_t st);
// two-waves-per-SIMD dK/dV kernel for the shapes dkdv_split_applies() accepts
bool dkdv_split_applies(const KArgs& a);
int launch_bwd_dkdv_split_bf16(const KArgs& a, hipStream_t st);   // a.ds_spill set: also stores the dS blobs
// dQ from the dS blobs the dK/dV kernel stored (same shapes as dkdv_split_applies)
int launch_bwd_dq_spill_bf16(const KArgs& a, hipStream_t st);

// delta[b,h,t] = sum_d dout[b,t,h,d] * o[b,t,h,d], fp32
int launch_delta(const KArgs& a, int dtype, hipStream_t st);
// dk = partial[class 0] + partial[class 1] (same for dv), cast to the output type
int launch_combine_partials(const KArgs& a, int dtype, hipStream_t st);

// Number of tile sequences walked together (see decode_slot) for a kernel whose XCD holds
// `slots` workgroups at a time, and the sequence count padded to a multiple of it.
inline int interleave_for(int T, int slots) { return T >= slots ? 1 : (slots + T - 1) / T; }
inline int pad_to(int n, int il) { return (n + il - 1) / il * il; }

}  // namespace s2
