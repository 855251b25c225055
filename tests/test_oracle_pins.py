"""Pins for the CPU oracle: every check here compares the oracle with something
other than itself - brute force over subsets, a hand-worked example, a closed
form the paper prints, Table 1's rounding, plain numpy routines, or an
invariant the method fixes.  CPU only."""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import des_oracle as O
from paper_2602_00879_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- brute force
def _best_subset(scores, allowed, k):
    """All k-subsets of `allowed`: maximal score sum, lexicographically smallest
    sorted tuple among equal sums (= lowest-index tie rule)."""
    best = None
    for comb in itertools.combinations(sorted(allowed), k):
        s = sum(scores[i] for i in comb)
        if best is None or s > best[0] or (s == best[0] and comb < best[1]):
            best = (s, comb)
    return set(best[1])


@pytest.mark.parametrize("seed", range(12))
def test_topk_equals_subset_enumeration(seed):
    rng = np.random.default_rng(seed)
    M = int(rng.integers(2, 9))
    K = int(rng.integers(1, M + 1))
    # small integers -> many exact ties; sums of integers are exact
    row = rng.integers(-3, 4, size=M).astype(np.float64)
    got = O.topk(row, K)
    assert set(got) == _best_subset(row, range(M), K)
    # rank order: non-increasing values, ties by ascending index
    for a, b in zip(got, got[1:]):
        assert (row[a] > row[b]) or (row[a] == row[b] and a < b)


@pytest.mark.parametrize("seed", range(12))
def test_constrained_topk_equals_subset_enumeration(seed):
    rng = np.random.default_rng(100 + seed)
    M = int(rng.integers(3, 9))
    core = sorted(rng.choice(M, size=int(rng.integers(1, M + 1)), replace=False).tolist())
    K = int(rng.integers(1, M + 1))
    row = rng.integers(-2, 3, size=M).astype(np.float64)
    got = O.constrained_topk(row, core, K)
    k_eff = min(K, len(core))
    assert len(got) == k_eff
    assert set(got) == _best_subset(row, core, k_eff)


@pytest.mark.parametrize("seed", range(10))
def test_vote_coreset_equals_subset_enumeration(seed):
    rng = np.random.default_rng(200 + seed)
    N, M = int(rng.integers(1, 6)), int(rng.integers(3, 9))
    K = int(rng.integers(1, M))
    C = int(rng.integers(1, M + 1))
    logits = rng.standard_normal((N, M))
    core, V, margin = O.coreset_vote(logits, K, C)
    # independent V: dense softmax times a 0/1 mask built from argsort
    P = np.exp(logits) / np.exp(logits).sum(1, keepdims=True)
    mask = np.zeros_like(P)
    for n in range(N):
        order = np.lexsort((np.arange(M), -logits[n]))
        mask[n, order[:K]] = 1.0
    V2 = (P * mask).sum(0)
    np.testing.assert_allclose(V, V2, rtol=1e-12, atol=0)
    nominated = [i for i in range(M) if mask[:, i].any()]
    c_eff = min(C, len(nominated))
    assert len(core) == c_eff
    assert set(core) == _best_subset(V2, nominated, c_eff)
    assert core == sorted(core)
    assert margin > 0


def test_vote_tie_goes_to_lowest_index():
    # two tokens, identical rows with exact ties between experts 1 and 2
    logits = np.array([[0.0, 1.0, 1.0, -1.0], [0.0, 1.0, 1.0, -1.0]])
    core, V, margin = O.coreset_vote(logits, K=2, C=1)
    assert V[1] == V[2]
    assert core == [1]
    assert margin == 0.0


# ---------------------------------------------------------- hand-worked example
def test_hand_worked_example():
    g = json.load(open(os.path.join(GOLD, "vote_3x5_worked_example.json")))
    P = np.array(g["probs"])
    logits = np.log(P)
    K, C = g["K"], g["C"]
    core, V, margin = O.coreset_vote(logits, K, C)
    np.testing.assert_allclose(V, g["votes"], rtol=1e-12, atol=1e-15)
    assert core == g["vote_coreset"]
    assert margin == pytest.approx(g["vote_margin"], rel=1e-12)
    r = O.route_block(logits, "vote", K, C)
    assert r["topk_idx"].tolist() == g["vote_topk_idx"]
    np.testing.assert_allclose(r["topk_w"], g["vote_gates"], rtol=1e-12)
    assert O.coreset_seq(logits, 1) == g["seq_k1_coreset"]
    assert O.coreset_seq(logits, 2) == g["seq_k2_coreset"]
    assert O.route_block(logits, "seq", K, 5, k_seq=1)["topk_idx"].tolist() == g["seq_k1_topk_idx"]
    rv = O.route_block(logits, "vanilla", K, 5)
    assert rv["topk_idx"].tolist() == g["vanilla_topk_idx"]
    # counts / unique experts through the layer entry point (weights irrelevant)
    D, F, M = 4, 2, 5
    z = np.zeros
    out = O.moe_forward(z((1, 3, D)), z((M, D)), None, z((M, F, D)), z((M, F, D)), z((M, D, F)),
                        K, C, "vote", logits_override=logits[None])
    assert out["counts"].tolist() == g["vote_counts"]
    out = O.moe_forward(z((1, 3, D)), z((M, D)), None, z((M, F, D)), z((M, F, D)), z((M, D, F)),
                        K, C, "vanilla", logits_override=logits[None])
    assert out["n_unique"] == g["vanilla_n_unique"]


# ------------------------------------------------------------------ closed form
@pytest.mark.parametrize("M,K,N", [(128, 8, 4), (128, 8, 32), (128, 8, 128), (256, 8, 32)])
def test_expected_unique_experts_uniform_routing(M, K, N):
    """Sec. 3: E|union S_n| = M(1-(1-K/M)^N) under uniform routing.  i.i.d.
    Gaussian logits make every token's top-K a uniform random K-subset."""
    seeds = 200
    tot = 0
    for s in range(seeds):
        L = W.make_logits(N, M, seed=1000 + s)
        r = O.moe_forward(np.zeros((1, N, 1)), np.zeros((M, 1)), None, None, None, None,
                          K, M, "vanilla", logits_override=L[None], compute_y=False)
        tot += r["n_unique"]
    mean = tot / seeds
    expect = O.expected_unique_uniform(M, K, N)
    # printed values for the 128-expert shape (derived from the formula)
    if (M, K) == (128, 8):
        assert expect == pytest.approx({4: 29.1, 32: 111.8, 128: 128.0}[N], abs=0.06)
    # per-sample std is below sqrt(M)/2; 5 sigma of the mean
    tol = 5 * (math.sqrt(M) / 2) / math.sqrt(seeds) + 0.05
    assert abs(mean - expect) < tol, (mean, expect)


def test_beta_rounding_matches_table1():
    # Table 1: beta=0.15 -> 38 and 0.10 -> 25 (256-expert model);
    #          beta=0.6 -> 38 and 0.4 -> 25 (64-expert model)
    assert O.coreset_size_from_beta(0.15, 256) == 38
    assert O.coreset_size_from_beta(0.10, 256) == 25
    assert O.coreset_size_from_beta(0.6, 64) == 38
    assert O.coreset_size_from_beta(0.4, 64) == 25
    # the other roundings would contradict the table
    assert round(0.10 * 256) == 26 and math.ceil(0.15 * 256) == 39


# ------------------------------------------------------- FFN / combine reductions
def _rand_layer(rng, B, N, D, M, F, shared=False):
    x = rng.standard_normal((B, N, D))
    wr = rng.standard_normal((M, D)) * 0.3
    wg = rng.standard_normal((M, F, D)) * 0.2
    wu = rng.standard_normal((M, F, D)) * 0.2
    wd = rng.standard_normal((M, D, F)) * 0.2
    sh = None
    if shared:
        sh = (rng.standard_normal((F + 1, D)) * 0.2, rng.standard_normal((F + 1, D)) * 0.2,
              rng.standard_normal((D, F + 1)) * 0.2)
    return x, wr, wg, wu, wd, sh


def test_single_expert_is_plain_swiglu_mlp():
    rng = np.random.default_rng(7)
    x, wr, wg, wu, wd, _ = _rand_layer(rng, 1, 5, 12, 1, 9)
    out = O.moe_forward(x, wr, None, wg, wu, wd, K=1, C=1, mode="vanilla")
    X = x[0]
    G = X @ wg[0].T
    H = (G / (1 + np.exp(-G))) * (X @ wu[0].T)
    np.testing.assert_allclose(out["y"][0], H @ wd[0].T, rtol=1e-12, atol=1e-14)
    assert np.all(out["topk_w"] == 1.0)


@pytest.mark.parametrize("mode", ["vanilla", "seq", "vote"])
def test_layer_equals_dense_one_hot_einsum(mode):
    rng = np.random.default_rng(11)
    B, N, D, M, F, K, C = 2, 6, 10, 7, 5, 3, 4
    x, wr, wg, wu, wd, sh = _rand_layer(rng, B, N, D, M, F, shared=True)
    bias = rng.standard_normal(M)
    out = O.moe_forward(x, wr, bias, wg, wu, wd, K, C, mode, shared=sh, residual=True)
    # dense: every expert for every token, times a gate matrix rebuilt from
    # probabilities restricted to the selected set (Eq. 1's normalisation)
    G = np.einsum("bnd,mfd->bnmf", x, wg)
    U = np.einsum("bnd,mfd->bnmf", x, wu)
    E = np.einsum("bnmf,mdf->bnmd", G / (1 + np.exp(-G)) * U, wd)
    L = np.einsum("bnd,md->bnm", x, wr) + bias
    P = np.exp(L) / np.exp(L).sum(-1, keepdims=True)
    gate = np.zeros((B, N, M))
    for b in range(B):
        for n in range(N):
            S = [e for e in out["topk_idx"][b, n] if e >= 0]
            gate[b, n, S] = P[b, n, S] / P[b, n, S].sum()
    y = np.einsum("bnm,bnmd->bnd", gate, E)
    Gs = x @ sh[0].T
    y = y + (Gs / (1 + np.exp(-Gs)) * (x @ sh[1].T)) @ sh[2].T + x
    np.testing.assert_allclose(out["y"], y, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(out["logits"], L, rtol=1e-12, atol=1e-13)


def test_output_is_linear_in_down_projection():
    rng = np.random.default_rng(13)
    x, wr, wg, wu, wd, _ = _rand_layer(rng, 1, 4, 8, 5, 6)
    a = O.moe_forward(x, wr, None, wg, wu, wd, 2, 3, "vote")["y"]
    b = O.moe_forward(x, wr, None, wg, wu, 3.0 * wd, 2, 3, "vote")["y"]
    np.testing.assert_allclose(b, 3.0 * a, rtol=1e-12)


# ------------------------------------------------------------------- invariants
@pytest.mark.parametrize("mode", ["vanilla", "seq", "vote"])
@pytest.mark.parametrize("seed", range(6))
def test_invariants_random(mode, seed):
    rng = np.random.default_rng(300 + seed)
    N, M = int(rng.integers(1, 20)), int(rng.integers(2, 40))
    K = int(rng.integers(1, min(M, 8) + 1))
    C = int(rng.integers(1, M + 1))
    L = rng.standard_normal((N, M)).astype(np.float32)
    r = O.route_block(L, mode, K, C)
    core = r["coreset"]
    assert core == sorted(set(core))
    if mode != "vanilla":
        assert len(core) <= C
    k_eff = min(K, len(core))
    for n in range(N):
        S = [e for e in r["topk_idx"][n] if e >= 0]
        assert len(S) == k_eff and len(set(S)) == k_eff
        assert set(S) <= set(core)                      # Alg. 1: routed inside the coreset
        assert r["topk_w"][n].sum() == pytest.approx(1.0, abs=1e-12)
        assert np.all(r["topk_idx"][n, k_eff:] == -1) and np.all(r["topk_w"][n, k_eff:] == 0)
    # the coreset does not depend on the order of the tokens
    perm = rng.permutation(N)
    assert O.route_block(L[perm], mode, K, C)["coreset"] == core


def test_vanilla_is_standard_topk_and_degenerate_modes_reduce_to_it():
    rng = np.random.default_rng(5)
    N, M, K = 9, 24, 4
    L = rng.standard_normal((N, M)).astype(np.float32)
    van = O.route_block(L, "vanilla", K, M)
    for n in range(N):
        order = np.lexsort((np.arange(M), -L[n].astype(np.float64)))
        assert van["topk_idx"][n].tolist() == order[:K].tolist()
    # vote with C >= M keeps every nominated expert -> same routing as vanilla
    vote = O.route_block(L, "vote", K, M)
    assert np.array_equal(vote["topk_idx"], van["topk_idx"])
    np.testing.assert_allclose(vote["topk_w"], van["topk_w"], rtol=0, atol=0)
    # seq with k_seq = K: the union of vanilla selections (Eq. 5 with k = K)
    seq = O.route_block(L, "seq", K, M, k_seq=K)
    assert np.array_equal(seq["topk_idx"], van["topk_idx"])
    assert seq["coreset"] == sorted(set(van["topk_idx"].reshape(-1).tolist()))
    # a single token with C = K elects exactly its own top-K
    one = O.route_block(L[:1], "vote", K, K)
    assert np.array_equal(one["topk_idx"], van["topk_idx"][:1])


def test_identical_tokens_give_vanilla_output():
    rng = np.random.default_rng(17)
    x, wr, wg, wu, wd, _ = _rand_layer(rng, 1, 1, 8, 9, 4)
    x = np.repeat(x, 5, axis=1)
    a = O.moe_forward(x, wr, None, wg, wu, wd, 3, 9, "vanilla")
    for mode in ("seq", "vote"):
        b = O.moe_forward(x, wr, None, wg, wu, wd, 3, 3, mode)
        assert np.array_equal(a["topk_idx"], b["topk_idx"])
        np.testing.assert_allclose(a["y"], b["y"], rtol=1e-13)


def test_seq_cap_rule():
    rng = np.random.default_rng(23)
    N, M, K = 12, 30, 5
    L = rng.standard_normal((N, M))
    sizes = [len(O.coreset_seq(L, k)) for k in range(1, K + 1)]
    assert sizes == sorted(sizes)                        # monotone in k'
    for C in (sizes[0], sizes[2], sizes[-1], sizes[1] + 1 if sizes[1] + 1 < sizes[2] else sizes[1]):
        core, used = O.coreset_seq_capped(L, K, C)
        assert used >= 1 and len(core) <= C
        assert core == O.coreset_seq(L, used)
        assert used == K or len(O.coreset_seq(L, used + 1)) > C
    # overflow: fewer slots than distinct top-1 experts
    C = sizes[0] - 1
    if C >= 1:
        core, used = O.coreset_seq_capped(L, K, C)
        assert used == 0 and len(core) == C
        top1 = [int(np.argmax(L[n])) for n in range(N)]
        nom = {e: top1.count(e) for e in set(top1)}
        assert set(core) <= set(top1)
        worst_in = min(nom[e] for e in core)
        assert all(nom[e] <= worst_in for e in set(top1) - set(core))


def test_counts_and_unique():
    rng = np.random.default_rng(29)
    x, wr, wg, wu, wd, _ = _rand_layer(rng, 3, 7, 6, 11, 3)
    out = O.moe_forward(x, wr, None, wg, wu, wd, 4, 5, "vote", compute_y=False)
    k_eff = [min(4, len(c)) for c in out["coresets"]]
    assert out["counts"].sum() == sum(7 * k for k in k_eff)
    assert out["n_unique"] == (out["counts"] > 0).sum()
    assert out["n_unique"] <= len(set().union(*map(set, out["coresets"])))


def test_stack_is_residual_composition():
    rng = np.random.default_rng(31)
    layers = []
    for _ in range(3):
        x, wr, wg, wu, wd, _ = _rand_layer(rng, 2, 4, 6, 5, 3)
        layers.append(dict(w_router=wr, bias=None, w_gate=wg, w_up=wu, w_down=wd))
    y, per = O.moe_stack_forward(x, layers, 2, 3, "vote")
    cur = x
    for lw in layers:
        cur = cur + O.moe_forward(cur, lw["w_router"], None, lw["w_gate"], lw["w_up"],
                                  lw["w_down"], 2, 3, "vote")["y"]
    np.testing.assert_allclose(y, cur, rtol=1e-13)


# ------------------------------------------------------------ input generators
def test_bf16_rounding_is_nearest_even():
    a = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.1415927], dtype=np.float32)
    bits = W.f32_to_bf16_bits(a)
    back = W.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even mantissa (1.0);
    # 1 + 3*2^-8 is a tie -> rounds up to 1 + 2^-6 (even)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625)
    assert back[3] == -2.5
    assert abs(back[4] - a[4]) <= 2.0 ** -7
    import torch
    t = torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    assert np.array_equal(t, back)


def test_workload_shapes_and_seeding():
    cfg = W.CONFIGS["tiny_f32"]
    a, b = W.make_layer(cfg), W.make_layer(cfg)
    assert a["x"].shape == (1, 8, 256) and a["w_router"].shape == (16, 256)
    assert a["w_gate"].shape == (16, 128, 256) and a["w_down"].shape == (16, 256, 128)
    assert np.array_equal(a["w_up"], b["w_up"])
    assert abs(float(a["w_gate"].std()) - 0.02) < 1e-3
    zb = W.zipf_bias(128, 1.1, np.random.default_rng(0))
    assert abs(float(zb.mean())) < 1e-5 and sorted(-zb)[1] - sorted(-zb)[0] == pytest.approx(1.1 * math.log(2), rel=1e-5)


# ------------------------------------------- routing variants (Sec. 5.1 / 5.3)
def test_cumulative_skip_hand_values():
    """Sec. 5.1 (Baselines): experts i..K are skipped when their cumulative
    probability is below beta of the total.  Gates 0.5 / 0.3 / 0.15 / 0.05:
    beta = 0.1 -> only the last (0.05 < 0.1, but 0.05 + 0.15 = 0.2 is not);
    beta = 0.25 -> the last two (0.2 < 0.25, 0.5 is not); beta = 0.6 -> three
    (0.5 < 0.6); the best expert always stays."""
    g = np.array([0.5, 0.3, 0.15, 0.05])
    assert O.cumulative_skip(g, 0.0)[0] == 4
    assert O.cumulative_skip(g, 0.1)[0] == 3
    assert O.cumulative_skip(g, 0.25)[0] == 2
    assert O.cumulative_skip(g, 0.6)[0] == 1
    assert O.cumulative_skip(g, 0.999)[0] == 1
    # scale invariance: "relative to the total routing sum"
    assert O.cumulative_skip(7.0 * g, 0.25)[0] == 2
    # the reported margin is the distance of the closest cut to the threshold
    assert O.cumulative_skip(g, 0.1)[1] == pytest.approx(0.05)


@pytest.mark.parametrize("seed", range(10))
def test_cumulative_skip_equals_enumeration_of_cuts(seed):
    rng = np.random.default_rng(100 + seed)
    k = int(rng.integers(1, 9))
    g = np.sort(rng.random(k))[::-1].copy()
    beta = float(rng.random()) * 0.9
    total = g.sum()
    valid = [i for i in range(1, k) if g[i:].sum() < beta * total]   # every admissible cut
    want = min(valid) if valid else k                                  # the largest skipped suffix
    keep, _ = O.cumulative_skip(g, beta)
    assert keep == want
    # monotone: a larger threshold never keeps more
    assert O.cumulative_skip(g, min(0.95, beta + 0.05))[0] <= keep


def test_k_route_keeps_the_coreset_and_truncates_each_token():
    """Sec. 5.3 (effect of active expert count): same coreset, fewer experts per
    token.  The election is unchanged, each token keeps the first k_route of
    its K coreset experts (rank order), gates are normalised over those."""
    L = W.make_logits(24, 40, seed=5, zipf_s=1.1)
    full = O.route_block(L, "vote", 8, 12)
    half = O.route_block(L, "vote", 8, 12, k_route=4)
    assert half["coreset"] == full["coreset"]
    assert np.array_equal(half["topk_idx"][:, :4], full["topk_idx"][:, :4])
    assert np.all(half["topk_idx"][:, 4:] == -1) and np.all(half["topk_w"][:, 4:] == 0)
    np.testing.assert_allclose(half["topk_w"].sum(axis=1), 1.0, atol=1e-12)
    ratio = full["topk_w"][:, :4] / full["topk_w"][:, :4].sum(axis=1, keepdims=True)
    np.testing.assert_allclose(half["topk_w"][:, :4], ratio, atol=1e-12)
    # k_route = K is the default path
    same = O.route_block(L, "vote", 8, 12, k_route=8)
    assert np.array_equal(same["topk_idx"], full["topk_idx"])
    # without a coreset, k_route = k is plain top-k routing (Table 1's "top-k" baseline)
    van = O.route_block(L, "vanilla", 8, 40, k_route=4)
    top4 = O.route_block(L, "vanilla", 4, 40)
    assert np.array_equal(van["topk_idx"][:, :4], top4["topk_idx"])
    np.testing.assert_allclose(van["topk_w"][:, :4], top4["topk_w"], atol=1e-12)


def test_skip_in_route_block():
    L = W.make_logits(16, 32, seed=9, zipf_s=1.1, scale=2.0)
    base = O.route_block(L, "vanilla", 6, 32)
    skp = O.route_block(L, "vanilla", 6, 32, skip_beta=0.15)
    kept = (skp["topk_idx"] >= 0).sum(axis=1)
    assert kept.min() >= 1 and kept.max() <= 6 and kept.min() < 6   # something was skipped
    for n in range(16):
        k = int(kept[n])
        assert np.array_equal(skp["topk_idx"][n, :k], base["topk_idx"][n, :k])
        g = base["topk_w"][n]
        assert g[k:].sum() < 0.15 * g.sum() or k == 6                # the dropped tail is below beta
        if k > 1:
            assert g[k - 1:].sum() >= 0.15 * g.sum()                 # and no longer tail would be
        np.testing.assert_allclose(skp["topk_w"][n, :k], g[:k] / g[:k].sum(), atol=1e-12)
    assert skp["skip_margin"] > 0


# ------------------------------------------- other routers (Sec. 4.1, sigma)
def test_sigmoid_router_and_renormalised_votes():
    """A sigma other than softmax (Sec. 4.1 leaves it to the model): with a sigmoid router the weights are
    logistic scores; rankings (and therefore DES-Seq and every top-K) do not
    change because the sigmoid is monotone; votes and gates do."""
    L = W.make_logits(20, 24, seed=3, zipf_s=0.7, scale=1.5)
    # closed forms on hand values
    np.testing.assert_allclose(O.router_scores(np.array([[0.0, np.log(3.0)]]), "sigmoid"), [[0.5, 0.75]])
    np.testing.assert_allclose(O.gates([0.0, np.log(3.0), 5.0], [1, 0], "sigmoid"), [0.6, 0.4])
    # votes: brute-force double loop over (token, expert) with an explicit mask
    for act in ("softmax", "sigmoid"):
        S = O.router_scores(L, act)
        for renorm in (False, True):
            V, nominated = O.vote_vector(L, 5, act, renorm)
            want = np.zeros(24)
            for n in range(20):
                order = sorted(range(24), key=lambda i: (-L[n, i], i))[:5]
                tot = sum(S[n, i] for i in order)
                for i in order:
                    want[i] += S[n, i] / (tot if renorm else 1.0)
            np.testing.assert_allclose(V, want, rtol=1e-13)
            if renorm:   # every token casts a total weight of one
                assert V.sum() == pytest.approx(20.0)
    # monotone activation: DES-Seq and vanilla index decisions are unchanged
    for mode in ("vanilla", "seq"):
        a = O.route_block(L, mode, 5, 9)
        b = O.route_block(L, mode, 5, 9, act="sigmoid")
        assert a["coreset"] == b["coreset"] and np.array_equal(a["topk_idx"], b["topk_idx"])
        assert not np.allclose(a["topk_w"], b["topk_w"])
        np.testing.assert_allclose(b["topk_w"].sum(axis=1), 1.0, atol=1e-12)
    # renormalised softmax votes = softmax over the K selected logits
    V, _ = O.vote_vector(L, 5, "softmax", True)
    want = np.zeros(24)
    for n in range(20):
        sel = O.topk(L[n], 5)
        for i, g in zip(sel, O.gates(L[n], sel)):
            want[i] += g
    np.testing.assert_allclose(V, want, rtol=1e-12)


# -------------------------------- group-limited routers (Sec. 4.1, sigma)
def test_group_limit_hand_worked():
    """Six experts in three groups of two, two groups kept.  The two group
    scores disagree on these numbers: by best member the groups score
    (0.90, 0.50, 0.60), by the sum of the two best (0.95, 0.99, 0.90)."""
    s = [0.90, 0.05, 0.50, 0.49, 0.60, 0.30]
    a, m = O.group_limited(s, 3, 2, "max")
    assert a == [True, True, False, False, True, True]
    assert m == pytest.approx((0.60 - 0.50) / 0.60)
    a, m = O.group_limited(s, 3, 2, "top2sum")
    assert a == [True, True, True, True, False, False]
    assert m == pytest.approx((0.95 - 0.90) / 0.95)
    # equal group scores: the lower group index is kept
    a, m = O.group_limited([1.0, 0.0, 0.0, 1.0, 0.5, 0.5], 3, 1, "max")
    assert a == [True, True, False, False, False, False] and m == 0.0
    # one group, or every group kept: no limit at all
    assert O.group_limited(s, 1, 1, "max") == ([True] * 6, math.inf)
    assert O.group_limited(s, 3, 3, "top2sum") == ([True] * 6, math.inf)
    for n_group, topk_group in ((4, 1), (3, 0), (3, 4)):
        with pytest.raises(ValueError):
            O.group_limited(s, n_group, topk_group, "max")


@pytest.mark.parametrize("seed", range(10))
def test_group_limit_against_a_scan_of_the_ranking_and_pair_enumeration(seed):
    """"max": walking the token's experts best first, the kept groups are the
    first topk_group distinct groups met.  "top2sum": a group's score is the
    largest sum over all pairs of its members (scores are positive), found here
    by enumerating the pairs; the kept groups are then found by enumerating
    every topk_group-subset of groups for the largest total."""
    rng = np.random.default_rng(100 + seed)
    n_group = int(rng.integers(2, 6))
    size = int(rng.integers(2, 5))
    topk_group = int(rng.integers(1, n_group))
    M = n_group * size
    s = rng.random(M) + 0.01
    if seed % 3 == 0:   # exact ties between groups
        s = np.round(s * 4) / 4 + 0.25
    allowed, _ = O.group_limited(s, n_group, topk_group, "max")
    seen = []
    for i in sorted(range(M), key=lambda i: (-s[i], i)):
        if i // size not in seen:
            seen.append(i // size)
    # equal best members: the lower group index first
    best = [max(s[g * size:(g + 1) * size]) for g in range(n_group)]
    seen.sort(key=lambda g: (-best[g], g))
    assert allowed == [(i // size) in seen[:topk_group] for i in range(M)]

    allowed, _ = O.group_limited(s, n_group, topk_group, "top2sum")
    pair = [max(s[i] + s[j] for i, j in itertools.combinations(range(g * size, (g + 1) * size), 2))
            for g in range(n_group)]
    want = _best_subset(pair, range(n_group), topk_group)
    assert allowed == [(i // size) in want for i in range(M)]


def test_group_limit_in_the_layer():
    L = W.make_logits(24, 64, seed=5, zipf_s=0.9, scale=1.5)
    K, C = 4, 6
    for act, kind in (("softmax", "max"), ("sigmoid", "top2sum")):
        S = O.router_scores(L, act)
        allowed = np.array([O.group_limited(S[n], 8, 2, kind)[0] for n in range(24)])
        # vanilla: the architecture's own routing = top-K of the allowed experts
        v = O.route_block(L, "vanilla", K, 64, act=act, n_group=8, topk_group=2, group_score=kind)
        for n in range(24):
            mine = [int(e) for e in v["topk_idx"][n]]
            assert all(allowed[n, e] for e in mine)
            assert len(set(e // 8 for e in mine)) <= 2
            masked = np.where(allowed[n], L[n], -1e30)      # plain masked top-K
            assert mine == [int(i) for i in np.argsort(-masked, kind="stable")[:K]]
        # votes: explicit double loop over allowed nominations
        V, nominated = O.vote_vector(L, K, act, False, allowed)
        want = np.zeros(64)
        for n in range(24):
            order = [i for i in sorted(range(64), key=lambda i: (-L[n, i], i)) if allowed[n, i]][:K]
            for i in order:
                want[i] += S[n, i]
        np.testing.assert_allclose(V, want, rtol=1e-13)
        # DES: every token stays inside coreset AND its own groups; a token may be short
        for mode in ("seq", "vote"):
            r = O.route_block(L, mode, K, C, act=act, n_group=8, topk_group=2, group_score=kind)
            core = set(r["coreset"])
            short = 0
            for n in range(24):
                mine = [int(e) for e in r["topk_idx"][n] if e >= 0]
                assert all(e in core and allowed[n, e] for e in mine)
                room = sum(1 for e in core if allowed[n, e])
                assert len(mine) == min(K, room)
                short += len(mine) < K
                if mine:
                    assert r["topk_w"][n].sum() == pytest.approx(1.0)
                else:
                    assert r["topk_w"][n].sum() == 0.0
            assert r["group_margin"] > 0
            assert short > 0     # the case this test is about does occur
    # no groups, one group, or all groups kept: identical to the unlimited layer
    base = O.route_block(L, "vote", K, C)
    for ng, tg in ((0, 0), (1, 1), (8, 8)):
        r = O.route_block(L, "vote", K, C, n_group=ng, topk_group=tg)
        assert r["coreset"] == base["coreset"] and np.array_equal(r["topk_idx"], base["topk_idx"])
        np.testing.assert_array_equal(r["topk_w"], base["topk_w"])


# ------------------------------------------------ attention around the MoE layers
def _attn_case(seed, B=2, N=5, D=12, H=4, Hkv=2, dh=3, P=6):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, N, D))
    wq = rng.standard_normal((H * dh, D)) * 0.4
    wk = rng.standard_normal((Hkv * dh, D)) * 0.4
    wv = rng.standard_normal((Hkv * dh, D)) * 0.4
    wo = rng.standard_normal((D, H * dh)) * 0.4
    kc = rng.standard_normal((B, Hkv, P, dh))
    vc = rng.standard_normal((B, Hkv, P, dh))
    return x, wq, wk, wv, wo, kc, vc, H, Hkv


@pytest.mark.parametrize("seed", range(4))
def test_block_attention_equals_library_attention(seed):
    """The oracle's loops against torch's scaled_dot_product_attention on the CPU (a library
    routine, float64): projections, grouped key/value heads, the window of cached and block
    positions, the scale 1/sqrt(dh), the output projection, the residual."""
    import torch
    x, wq, wk, wv, wo, kc, vc, H, Hkv = _attn_case(seed)
    B, N, D = x.shape
    dh = wq.shape[0] // H
    y = O.block_attention(x, wq, wk, wv, wo, kc, vc, H, Hkv, residual=True)
    tx = torch.from_numpy(x)
    q = (tx @ torch.from_numpy(wq).T).reshape(B, N, H, dh).permute(0, 2, 1, 3)
    k = (tx @ torch.from_numpy(wk).T).reshape(B, N, Hkv, dh).permute(0, 2, 1, 3)
    v = (tx @ torch.from_numpy(wv).T).reshape(B, N, Hkv, dh).permute(0, 2, 1, 3)
    keys = torch.cat([torch.from_numpy(kc), k], dim=2).repeat_interleave(H // Hkv, dim=1)
    vals = torch.cat([torch.from_numpy(vc), v], dim=2).repeat_interleave(H // Hkv, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(q, keys, vals)   # no mask, scale 1/sqrt(dh)
    ref = o.permute(0, 2, 1, 3).reshape(B, N, H * dh) @ torch.from_numpy(wo).T + tx
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)


def test_block_attention_invariants():
    """What the definition fixes whatever the numbers: (1) with all scores equal the weights
    are uniform, so a head's output is the mean of its values; (2) the result does not depend
    on the order of the cached positions; (3) with no cached position and a single block token
    the token attends to itself only; (4) sequences are independent; (5) adding one cached key
    of score 0 moves a head's output by p * (value - output) with p = 1 / (Z + 1)."""
    x, wq, wk, wv, wo, kc, vc, H, Hkv = _attn_case(7)
    B, N, D = x.shape
    dh = wq.shape[0] // H
    P = kc.shape[2]
    # (1) zero queries: every score is 0; cached values all equal c, block values 0 (wv = 0)
    c = np.arange(1, dh + 1, dtype=np.float64)
    y = O.block_attention(x, wq * 0.0, wk, np.zeros_like(wv), wo, kc, np.broadcast_to(c, vc.shape).copy(), H, Hkv)
    head = np.tile(c * P / (P + N), H)
    np.testing.assert_allclose(y, np.broadcast_to(head @ wo.T, y.shape), rtol=1e-12, atol=1e-12)
    # (2) permutation of the cache
    perm = np.random.default_rng(1).permutation(P)
    y0 = O.block_attention(x, wq, wk, wv, wo, kc, vc, H, Hkv)
    y1 = O.block_attention(x, wq, wk, wv, wo, kc[:, :, perm], vc[:, :, perm], H, Hkv)
    np.testing.assert_allclose(y0, y1, rtol=1e-12, atol=1e-13)
    # (3) one token, empty cache: y = wo [wv x, each query head reading its key/value group]
    x1 = x[:1, :1]
    e = np.zeros((1, Hkv, 0, dh))
    y3 = O.block_attention(x1, wq, wk, wv, wo, e, e, H, Hkv)
    v = wv @ x1[0, 0]
    heads = np.concatenate([v[(h // (H // Hkv)) * dh:(h // (H // Hkv) + 1) * dh] for h in range(H)])
    np.testing.assert_allclose(y3[0, 0], wo @ heads, rtol=1e-12, atol=1e-13)
    # (4) sequences are independent
    yb = O.block_attention(x[1:], wq, wk, wv, wo, kc[1:], vc[1:], H, Hkv)
    np.testing.assert_allclose(y0[1:], yb, rtol=1e-12, atol=1e-13)
    # (5) one more cached key with score 0 (a zero key) and value 1e6 in every coordinate;
    # an identity output projection exposes the heads
    kc5 = np.concatenate([kc, np.zeros((B, Hkv, 1, dh))], axis=2)
    vc5 = np.concatenate([vc, np.full((B, Hkv, 1, dh), 1e6)], axis=2)
    eye = np.eye(D, H * dh)
    y5 = O.block_attention(x, wq, wk, wv, eye, kc5, vc5, H, Hkv)
    y5_0 = O.block_attention(x, wq, wk, wv, eye, kc, vc, H, Hkv)
    h, n = 1, 2
    g = h // (H // Hkv)
    keys = np.concatenate([kc[0, g], (x[0] @ wk.T)[:, g * dh:(g + 1) * dh]], axis=0)
    s = keys @ (x[0] @ wq.T)[n, h * dh:(h + 1) * dh] / math.sqrt(dh)
    p_extra = 1.0 / (np.exp(s).sum() + 1.0)
    o_old = y5_0[0, n, h * dh:(h + 1) * dh]
    np.testing.assert_allclose(y5[0, n, h * dh:(h + 1) * dh], o_old + p_extra * (1e6 - o_old), rtol=1e-9)


def test_decoder_stack_is_the_two_sublayers_in_turn():
    """decoder_stack_forward against the two pinned sub-layers applied by hand, and the
    identity that zero attention output weights reduce it to the MoE stack."""
    rng = np.random.default_rng(5)
    B, N, D, M, F, K, C, H, Hkv, dh, P = 2, 4, 8, 6, 5, 2, 3, 2, 1, 4, 3
    layers = []
    for _ in range(3):
        layers.append(dict(
            wq=rng.standard_normal((H * dh, D)) * 0.3, wk=rng.standard_normal((Hkv * dh, D)) * 0.3,
            wv=rng.standard_normal((Hkv * dh, D)) * 0.3, wo=rng.standard_normal((D, H * dh)) * 0.3,
            k_cache=rng.standard_normal((B, Hkv, P, dh)), v_cache=rng.standard_normal((B, Hkv, P, dh)),
            w_router=rng.standard_normal((M, D)), bias=None, w_gate=rng.standard_normal((M, F, D)) * 0.3,
            w_up=rng.standard_normal((M, F, D)) * 0.3, w_down=rng.standard_normal((M, D, F)) * 0.3))
    x = rng.standard_normal((B, N, D))
    y, per = O.decoder_stack_forward(x, layers, K, C, "vote", H, Hkv)
    cur = x
    for lw in layers:
        a = cur + O.block_attention(cur, lw["wq"], lw["wk"], lw["wv"], lw["wo"], lw["k_cache"], lw["v_cache"], H, Hkv)
        cur = a + O.moe_forward(a, lw["w_router"], None, lw["w_gate"], lw["w_up"], lw["w_down"], K, C, "vote")["y"]
    np.testing.assert_allclose(y, cur, rtol=1e-12, atol=1e-12)
    zero = [dict(lw, wo=np.zeros_like(lw["wo"])) for lw in layers]
    y0, _ = O.decoder_stack_forward(x, zero, K, C, "vote", H, Hkv)
    y1, _ = O.moe_stack_forward(x, layers, K, C, "vote")
    np.testing.assert_allclose(y0, y1, rtol=1e-12, atol=1e-12)

