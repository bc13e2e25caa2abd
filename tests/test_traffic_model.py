"""The tile-schedule traffic model (paper_2410_09397_amd/traffic_model.py) against what fixes it from
outside: the oracle's replay of the four-phase scheme (which counts while it computes), the closed
forms and orders of the paper's I/O lemmas (App. C, App. D), and simple properties of this library's
own schedules."""
import numpy as np
import pytest

from oracle import attn_oracle as orc
from paper_2410_09397_amd import traffic_model as tm


@pytest.mark.parametrize("n,d,B", [(8, 4, 2), (9, 5, 3), (10, 4, 7), (6, 6, 16), (16, 8, 4)])
def test_small_cache_count_equals_the_replay(n, d, B):
    rng = np.random.default_rng(n * 100 + d)
    A1, A2, A3, dO = (0.4 * rng.standard_normal((n, d)) for _ in range(4))
    X, Y = 0.4 * rng.standard_normal((d, d)), 0.4 * rng.standard_normal((d, d))
    _, rd, wr = orc.small_cache_wgrad(A1, A2, A3, dO, X, Y, B)
    assert (rd, wr) == tm.paper_small_cache(n, d, B)


def test_small_cache_count_follows_thm_4_3():
    """reads = 12 (n^2 d + n d^2) / sqrt(M) + 6 n^2 + n with B = sqrt(M / 4) dividing n and d:
    O((n^2 d + n d^2) / sqrt(M)) as long as B <= d (M = o(d^2) is the regime of the theorem)."""
    for n, d, B in ((1024, 256, 16), (2048, 512, 32), (4096, 512, 64)):
        rd, _ = tm.paper_small_cache(n, d, B)
        M = 4 * B * B
        assert rd == 12 * (n * n * d + n * d * d) // int(np.sqrt(M)) + 6 * n * n + n
        # halving sqrt(M) doubles the leading term
        rd2, _ = tm.paper_small_cache(n, d, B // 2)
        lead, lead2 = rd - 6 * n * n - n, rd2 - 6 * n * n - n
        assert lead2 == 2 * lead


def test_large_cache_phase2_count_and_its_order():
    """The loops of phase 2 (App. D) move 4 n d + n + T_r 2 n d elements, T_r = ceil(n / B_r).  With
    B_r = M / 4d (M <= 4 d^2) that is 8 n^2 d^2 / M + O(n d): the Theta(n^2 d^2 / M) of Thm 4.1.
    Once M exceeds 4 d^2 the cap B_r <= d keeps the count at 2 n^2 instead of letting it fall
    further (the reading noted for this algorithm: the bound, not the count, is the yardstick)."""
    n, d = 4096, 128
    for M in (4 * d * 16, 4 * d * 64, 4 * d * d):
        rd, wr = tm.paper_large_cache_phase2(n, d, M)
        b_r = M // (4 * d)
        assert rd == 4 * n * d + n + (n // b_r) * 2 * n * d and wr == d * d
        assert abs(rd - (8 * n * n * d * d / M + 4 * n * d + n)) < 1e-6
    capped, _ = tm.paper_large_cache_phase2(n, d, 64 * d * d)
    assert capped == 4 * n * d + n + (n // d) * 2 * n * d  # = 2 n^2 + O(n d): no longer falls with M


def test_key_owner_streams_once_per_owned_block():
    n, d = 4096, 128
    a = tm.two_kernel(n, d, key_block=64, query_block=128, tile=64)
    # dQ owner: K, V once per 128-query block; dK/dV owner: Q, dO (+ LSE, v) once per 64-key block
    want = (n // 128) * 2 * n * d * 2 + (n // 64) * (2 * n * d * 2 + 2 * n * 4)
    assert a["streamed"] == want
    # doubling the owned blocks halves the streamed bytes; compulsory bytes stay
    b = tm.two_kernel(n, d, key_block=128, query_block=256, tile=64)
    assert b["streamed"] * 2 == a["streamed"]
    assert a["read"] - a["streamed"] == b["read"] - b["streamed"] == 5 * n * d * 2 + n * 4
    assert a["written"] == 3 * n * d * 2 + n * 4
    # the causal rule halves the streamed part up to the diagonal tiles
    c = tm.two_kernel(n, d, causal=True)
    assert 0.5 < c["streamed"] / a["streamed"] < 0.53


def test_one_pass_trades_recompute_for_atomic_bytes():
    n, d = 8192, 128
    two = tm.two_kernel(n, d, causal=True)
    for kb in (64, 128):
        one = tm.one_pass(n, d, causal=True, key_block=kb)
        # every visible (64-query tile, key block) pair adds a 64 x d fp32 tile
        tiles = sum(len(range((j0 // 64) * 64, n, 64)) for j0 in range(0, n, kb))
        assert one["atomics"] == tiles * 64 * d * 4
        assert one["written"] > 10 * two["written"]  # the additions dwarf every other byte written
    assert tm.one_pass(n, d, True, key_block=64)["atomics"] == 2 * tm.one_pass(n, d, True, key_block=128)["atomics"] - \
        (n // 128) * 64 * d * 4  # (the second half of a 128-key block skips one diagonal tile)


def test_four_phase_is_dominated_by_the_n_by_n_matrices():
    n, d = 4096, 512
    f = tm.four_phase(n, d)
    nn = n * n * 2
    assert f["written"] >= 2 * nn                       # f and p written once
    assert f["read"] >= 3 * nn                          # f read once, p twice
    large, small = tm.theorem_1_1_bytes(n, d, 160 * 1024)
    assert small < large                                # M = 160 KB < d^2 elements: the small-cache branch binds
    s = tm.split_d(n, d)
    assert s["streamed"] > f["streamed"]                # 32-row owners re-stream far more than 128 x 128 score tiles
