"""s2attn_bwd_ex_static (backward on the library's static device scratch, no workspace and
no allocation) against s2attn_bwd_ex on a caller workspace with the same (recomputing)
backward: same kernels on the same inputs, so the outputs must be identical.  Two calls in a row share the scratch array, the
second on a smaller problem."""
import numpy as np
import pytest

from paper_2309_12307_amd import inputs

pytestmark = pytest.mark.gpu


def run_both(shape, dtype, seed, **ex):
    import torch
    from gpu_util import to_dev
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D, G = shape
    bf = dtype == "bf16"
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=seed, dtype=dtype)
    q, k, v, do = (to_dev(inp[n], inp.get(n + "_bits") if bf else None) for n in ("q", "k", "v", "do"))
    o = torch.full_like(q, float("nan"))
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    binding.s2attn_fwd_ex(binding.make_params(q, k, v, o, lse, G, **ex))
    outs = []
    for static in (False, True):
        dq, dk, dv = (torch.full_like(t, float("nan")) for t in (q, k, v))
        if static:
            p = binding.make_params(q, k, v, o, lse, G, dout=do, dq=dq, dk=dk, dv=dv, **ex)
            binding.s2attn_bwd_ex_static(p)
        else:
            kw = dict(ex, bwd_algo=binding.BWD_RECOMPUTE)
            p = binding.make_params(q, k, v, o, lse, G, dout=do, dq=dq, dk=dk, dv=dv, **kw)
            ws = torch.empty(binding.bwd_workspace_bytes_ex(p), dtype=torch.uint8, device="cuda")
            p = binding.make_params(q, k, v, o, lse, G, dout=do, dq=dq, dk=dk, dv=dv, workspace=ws, **kw)
            binding.s2attn_bwd_ex(p)
        torch.cuda.synchronize()
        outs.append([t.float().cpu().numpy() for t in (dq, dk, dv)])
    return outs


CASES = [
    # (first call, second call on a smaller problem), dtype
    (((1, 4096, 8, 8, 128, 1024), (1, 1024, 4, 2, 128, 256)), "bf16"),     # aligned kernels, MHA then GQA
    (((1, 1536, 6, 3, 128, 512), (1, 400, 2, 1, 128, 200)), "bf16"),       # partial sums in the scratch, then unaligned MQA
    (((2, 512, 4, 2, 64, 128), (1, 256, 4, 4, 64, 64)), "f32"),
]


@pytest.mark.parametrize("shapes,dtype", CASES)
def test_static_scratch_backward_equals_workspace_backward(shapes, dtype):
    for n, shape in enumerate(shapes):
        ref, got = run_both(shape, dtype, seed=700 + n)
        for name, a, b in zip(("dq", "dk", "dv"), ref, got):
            assert np.all(np.isfinite(b)), (shape, name)
            assert np.array_equal(a, b), (shape, name, float(np.abs(a - b).max()))


def test_static_scratch_backward_matches_the_oracle_after_a_larger_call():
    """The second, smaller call must not see anything the first left in the scratch array:
    checked against the CPU oracle, not only against the other entry point."""
    from oracle import s2attn_oracle as orc
    from gpu_util import check_bf16_tensor
    run_both((1, 8192, 8, 8, 128, 2048), "bf16", seed=710)
    shape = (1, 768, 4, 2, 128, 256)
    B, N, H, Hkv, D, G = shape
    _, got = run_both(shape, "bf16", seed=711)
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=711, dtype="bf16")
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G)
    for name, g, r in zip(("dq", "dk", "dv"), got, ref[2:]):
        check_bf16_tensor(name, g, r)


def test_static_scratch_backward_refuses_what_does_not_fit():
    import torch
    from paper_2309_12307_amd import binding
    # B * H * N = 4 Mi rows need 32 MiB of row terms: over the 16 MiB array.  Refused on the host
    # before any pointer is looked at, so small dummy tensors are enough.
    t = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    p = binding.make_params(t, t, t, t, t, 8192, dout=t, dq=t, dk=t, dv=t, dims=(1, 131072, 32, 32, 128),
                            dtype=binding.BF16)
    with pytest.raises(binding.S2AttnError) as e:
        binding.s2attn_bwd_ex_static(p)
    assert e.value.code == -14


def test_forward_and_static_scratch_backward_replay_from_a_hip_graph():
    """The use the entry point is for: forward + backward captured once into a HIP graph (no
    allocation, no host synchronisation inside the calls) and replayed on new inputs, with
    eager work and synchronisations between the replays; every replay must equal the eager
    result bit for bit."""
    import torch
    from gpu_util import to_dev
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D, G = 1, 2048, 4, 2, 128, 512
    q, k, v, do = (torch.zeros((B, N, h, D), dtype=torch.bfloat16, device="cuda") for h in (H, Hkv, Hkv, H))
    o, dq = torch.zeros_like(q), torch.zeros_like(q)
    dk, dv = torch.zeros_like(k), torch.zeros_like(v)
    lse = torch.zeros((B, H, N), dtype=torch.float32, device="cuda")
    p_fwd = binding.make_params(q, k, v, o, lse, G)
    p_bwd = binding.make_params(q, k, v, o, lse, G, dout=do, dq=dq, dk=dk, dv=dv)

    def load(seed):
        inp = inputs.make_inputs(B, N, H, Hkv, D, seed=seed, dtype="bf16")
        for t, name in ((q, "q"), (k, "k"), (v, "v"), (do, "do")):
            t.copy_(to_dev(inp[name], inp[name + "_bits"]))

    def run():
        binding.s2attn_fwd_ex(p_fwd)
        binding.s2attn_bwd_ex_static(p_bwd)

    load(720)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                # warm-up outside the capture (device check, scratch address)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for seed in (721, 722, 723):
        load(seed)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (o, lse, dq, dk, dv)]
        for t in (o, lse, dq, dk, dv):
            t.fill_(float("nan"))
        run()                                # eager, same inputs
        torch.cuda.synchronize()
        for name, a, b in zip(("o", "lse", "dq", "dk", "dv"), got, (o, lse, dq, dk, dv)):
            assert torch.isfinite(a.float()).all(), (seed, name)
            assert torch.equal(a, b), (seed, name)
