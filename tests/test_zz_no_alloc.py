"""attn_bwd_noalloc (fixed device scratch inside the library) against attn_bwd (caller's workspace):
same kernels, so the same bits; two calls in a row, the second on a smaller input, which finds the
first call's leftovers in the scratch array."""
import pytest

from paper_2410_09397_amd import synth
from tests.helpers import to_dev

pytestmark = pytest.mark.gpu


def _case(w):
    import torch
    from paper_2410_09397_amd import attn
    inp = synth.make_inputs(w)
    Q, K, V, dO = (to_dev(inp[t], w.dtype) for t in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd(Q, K, V, w.scale, causal=w.causal)
    want = attn.attn_bwd(Q, K, V, O, dO, LSE, w.scale, causal=w.causal)
    got = tuple(torch.full_like(Q, float("nan")) for _ in range(3))
    attn.attn_bwd_noalloc(Q, K, V, O, dO, LSE, w.scale, got, causal=w.causal)
    torch.cuda.synchronize()
    for name, a, b in zip(("dQ", "dK", "dV"), got, want):
        assert torch.equal(a, b), (w.name, name)


def test_noalloc_matches_attn_bwd_twice_second_smaller():
    print("case noalloc bf16 d128 then a smaller d64 problem", flush=True)
    _case(synth.Workload("noalloc_a", 201, 2, 3, 700, 128, "bf16", causal=True))
    _case(synth.Workload("noalloc_b", 202, 1, 2, 130, 64, "bf16"))
    # the generic fp32 kernels and the four-phase path take their scratch from the same array
    _case(synth.Workload("noalloc_c", 203, 1, 2, 77, 40, "f32", causal=True))
    _case(synth.Workload("noalloc_d", 204, 1, 1, 200, 512, "bf16"))


def test_noalloc_call_captured_in_a_hip_graph_replays_like_eager_calls():
    """What the entry point is for: a caller under stream capture.  One eager call first (kernel attributes and the
    scratch address are looked up outside the capture), then the call is recorded once and replayed three times on
    new inputs, with the program's own eager work and synchronisations in between; every replay must give the bits
    of an eager attn_bwd on the same inputs."""
    import torch
    from paper_2410_09397_amd import attn

    def fresh(seed):
        inp = synth.make_inputs(synth.Workload("noalloc_graph", seed, 2, 4, 1000, 128, "bf16", causal=True))
        return [to_dev(inp[t], "bf16") for t in ("Q", "K", "V", "dO")]

    print("case noalloc under graph capture, bf16 d128 causal n1000", flush=True)
    scale = 128 ** -0.5
    Q, K, V, dO = fresh(301)
    O, LSE = attn.attn_fwd(Q, K, V, scale, causal=True)
    out = tuple(torch.zeros_like(Q) for _ in range(3))
    attn.attn_bwd_noalloc(Q, K, V, O, dO, LSE, scale, out, causal=True)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        attn.attn_bwd_noalloc(Q, K, V, O, dO, LSE, scale, out, causal=True)
    torch.cuda.synchronize()
    for seed in (302, 303, 304):
        for dst, src in zip((Q, K, V, dO), fresh(seed)):
            dst.copy_(src)
        o2, l2 = attn.attn_fwd(Q, K, V, scale, causal=True)
        O.copy_(o2)
        LSE.copy_(l2)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = attn.attn_bwd(Q, K, V, O, dO, LSE, scale, causal=True)
        torch.cuda.synchronize()
        for name, a, b in zip(("dQ", "dK", "dV"), out, want):
            assert torch.equal(a, b), (seed, name)


def test_noalloc_rejects_what_does_not_fit():
    import torch
    from paper_2410_09397_amd import attn
    # 3 Mi rows of 4 bytes exceed the 8 MiB array: the call is refused before anything is launched
    x = torch.zeros(1, 3, 1 << 20, 64, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(1, 3, 1 << 20, dtype=torch.float32, device="cuda")
    with pytest.raises(attn.AttnError) as e:
        attn.attn_bwd_noalloc(x, x, x, x, x, lse, 1.0, (x, x, x))
    assert e.value.status == attn.ATTN_ERR_WORKSPACE
