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


def test_noalloc_rejects_what_does_not_fit():
    import torch
    from paper_2410_09397_amd import attn
    # 3 Mi rows of 4 bytes exceed the 8 MiB array: the call is refused before anything is launched
    x = torch.zeros(1, 3, 1 << 20, 64, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(1, 3, 1 << 20, dtype=torch.float32, device="cuda")
    with pytest.raises(attn.AttnError) as e:
        attn.attn_bwd_noalloc(x, x, x, x, x, lse, 1.0, (x, x, x))
    assert e.value.status == attn.ATTN_ERR_WORKSPACE
