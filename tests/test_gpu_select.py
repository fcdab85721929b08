"""dmoe_select on the GPU against the oracle: masks, counts, offsets and lists must agree
bit-exactly (lists as sets; the library additionally promises ascending order)."""
import numpy as np
import pytest

from paper_2310_04361_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2310_04361_amd import binding
    binding.lib()
    return binding


def _check(B, oracle, scores, tau):
    import torch
    T, E = scores.shape
    tau32 = float(np.float32(tau))
    out = B.dmoe_select(torch.from_numpy(scores).cuda(), tau32)
    torch.cuda.synchronize()
    ref_mask, ref_k = oracle.select(scores.astype(np.float64), tau32)
    ref_counts, ref_offsets, ref_lists = oracle.bucket(ref_mask)
    got_mask = B.mask_bits_to_bool(out["mask_bits"], E)
    assert np.array_equal(got_mask, ref_mask)
    # bits beyond E stay clear
    words = out["mask_bits"].cpu().numpy().view(np.uint64)
    if E % 64:
        assert not (words[:, -1] >> np.uint64(E % 64)).any()
    assert np.array_equal(out["k_per_token"].cpu().numpy(), ref_k)
    assert np.array_equal(out["counts"].cpu().numpy(), ref_counts)
    offsets = out["offsets"].cpu().numpy()
    assert np.array_equal(offsets, ref_offsets)
    lists = out["token_lists"].cpu().numpy()[: offsets[-1]]
    for e in range(E):
        got = lists[offsets[e]:offsets[e + 1]]
        assert set(got.tolist()) == set(ref_lists[ref_offsets[e]:ref_offsets[e + 1]].tolist())
        assert (np.diff(got) > 0).all()
    return ref_mask


@pytest.mark.parametrize("T,E", [(1, 16), (63, 16), (64, 128), (65, 32), (257, 24), (1000, 128),
                                 (700, 256), (130, 70), (4099, 128),
                                 (12, 4096), (100, 2100), (17, 1), (16, 3), (70, 4096)])
@pytest.mark.parametrize("kind", ["halfnormal", "grid", "zipf"])
def test_select_matches_oracle(B, oracle, T, E, kind):
    scores = wl.random_scores(T, E, seed=T + E, kind=kind)
    for tau in (0.0, 0.25, 0.5, 0.9, 1.0):
        print(f"select T={T} E={E} kind={kind} tau={tau}", flush=True)
        _check(B, oracle, scores, tau)


def test_select_degenerate_rows(B, oracle):
    scores = wl.random_scores(200, 64, seed=9)
    scores[3] = 0.0                 # all-zero row: every expert passes 0 >= tau * 0
    scores[7] = 2.5                 # all-equal row
    scores[11, :] = 0.0
    scores[11, 5] = 1.0             # one-hot row
    scores[13] = np.float32(1e-38)  # tiny values: tau * max stays exact in fp64
    scores[17] = np.float32(3e38)
    for tau in (0.0, 0.5, 1.0):
        m = _check(B, oracle, scores, tau)
        assert m[3].all() and m[7].all()
        if tau > 0:
            assert m[11].sum() == 1


def test_select_exact_threshold_in_fp32(B, oracle):
    """Scores whose fp32 product tau * max would round across the threshold: the rule is the
    exact real comparison, so the fp64 oracle and the GPU must still agree."""
    rng = np.random.default_rng(5)
    mx = rng.uniform(1, 2, size=(512, 1)).astype(np.float32)
    tau = np.float32(0.3)
    exact = mx.astype(np.float64) * float(tau)
    near = np.nextafter(exact.astype(np.float32), np.float32(0))     # just below / at
    s = np.concatenate([mx, exact.astype(np.float32), near, np.nextafter(near, np.float32(4))] * 4, axis=1)
    _check(B, oracle, np.ascontiguousarray(s), float(tau))


def test_select_empty(B):
    import torch
    out = B.dmoe_select(torch.zeros((0, 16), dtype=torch.float32, device="cuda"), 0.5)
    torch.cuda.synchronize()
    assert out["offsets"].cpu().numpy().tolist() == [0] * 17
    assert out["counts"].cpu().numpy().tolist() == [0] * 16


# ---- the top-k gate ------------------------------------------------------------------------------
def _check_topk(B, oracle, scores, k):
    import torch
    T, E = scores.shape
    out = B.dmoe_select_topk(torch.from_numpy(scores).cuda(), k)
    torch.cuda.synchronize()
    ref_mask = oracle.select_topk(scores.astype(np.float64), k)
    ref_counts, ref_offsets, ref_lists = oracle.bucket(ref_mask)
    got_mask = B.mask_bits_to_bool(out["mask_bits"], E)
    assert np.array_equal(got_mask, ref_mask)          # bit-exact, ties included
    words = out["mask_bits"].cpu().numpy().view(np.uint64)
    if E % 64:
        assert not (words[:, -1] >> np.uint64(E % 64)).any()
    assert (out["k_per_token"].cpu().numpy() == k).all()
    assert np.array_equal(out["counts"].cpu().numpy(), ref_counts)
    offsets = out["offsets"].cpu().numpy()
    assert np.array_equal(offsets, ref_offsets) and offsets[-1] == T * k
    lists = out["token_lists"].cpu().numpy()[: offsets[-1]]
    for e in range(E):
        got = lists[offsets[e]:offsets[e + 1]]
        assert got.tolist() == ref_lists[ref_offsets[e]:ref_offsets[e + 1]].tolist()


@pytest.mark.parametrize("T,E", [(1, 16), (65, 32), (257, 24), (1000, 128), (300, 256), (130, 70),
                                 (40, 700), (4099, 128), (9, 4096), (70, 2100)])
@pytest.mark.parametrize("kind", ["halfnormal", "grid", "zipf"])
def test_select_topk_matches_oracle(B, oracle, T, E, kind):
    scores = wl.random_scores(T, E, seed=T + E + 1, kind=kind)   # "grid" is full of ties
    for k in sorted({0, 1, 2, E // 3, E - 1, E}):
        print(f"select_topk T={T} E={E} kind={kind} k={k}", flush=True)
        _check_topk(B, oracle, scores, k)


def test_select_topk_degenerate_rows(B, oracle):
    scores = wl.random_scores(100, 64, seed=11)
    scores[3] = 0.0                     # all equal: the k lowest indices
    scores[5] = -scores[5]              # negative scores are ordered as numbers
    scores[7, ::2] = np.float32(-0.0)   # -0 and +0 tie
    scores[7, 1::2] = 0.0
    for k in (1, 5, 64):
        _check_topk(B, oracle, scores, k)


def test_select_topk_rejects_bad_k(B):
    import torch
    s = torch.zeros((4, 16), dtype=torch.float32, device="cuda")
    for k in (-1, 17):
        with pytest.raises(B.DmoeError) as ei:
            B.dmoe_select_topk(s, k)
        assert ei.value.code == B.DMOE_ERR_SHAPE
