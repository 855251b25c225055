"""CPU oracle for one MoE layer under Dynamic Expert Sharing (DES).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP path is checked against.  Only the tests, the smoke entry and the
benchmark's cpu_baseline leg may import it; the product path never does.  It
shares no code with the HIP path and imports nothing from the package.

Everything is numpy in float64 on the exact input values (bf16 / fp32 inputs
are upcast by the caller; nothing is rounded in here).  Each function follows
one passage of the paper:

  router_logits        Background (efficient MoE): the router G maps R^D to R^M
  softmax_rows         Sec. 4.3 (per-token softmax of the selection kernel)
  router_scores        the routing function sigma, which Sec. 4.1 leaves to the model:
                       softmax over the experts, or a per-expert sigmoid
  rank_order           TopK of Eq. 1: the K experts with the best scores
  group_limited        group-limited routers (another sigma of Sec. 4.1): the groups of
                       experts a token may choose from
  coreset_seq          Eq. 5 / Alg. 2  (DES-Seq)
  coreset_vote         Eq. 6 / Alg. 3  (DES-Vote)
  constrained_topk     Alg. 1, stage 2, S_n
  cumulative_skip      Sec. 5.1, Baselines: the adapted NAEE rule (skip the bottom
                       experts whose cumulative probability is below beta)
  gates                Alg. 1, stage 2, g_n   (sigma = softmax, i.e. Eq. 1's
                       normalisation by the selected sum)
  expert_ffn           E_i(x): SwiGLU sub-network (form fixed by the workload)
  moe_forward          Alg. 1 as a whole (+ Eq. 1 when mode == "vanilla")
  moe_stack_forward    residual stack of such layers
  block_attention      the attention sub-layer around the MoE layers in a decoding step
                       (Fig. 2 left names its share of the latency; Sec. 5.1 fixes the
                       window: the block plus cached prefix and suffix positions)
  decoder_stack_forward     x <- x + Attn_l(x); x <- x + MoE_l(x), layer by layer
  expected_unique_uniform   closed form of Sec. 3 (Motivation)
  coreset_size_from_beta    M_core = beta * M (Sec. 5.1), floor (Table 1)

Readings taken where the paper is silent (each is listed with its reason in
the design notes of the repository):
  * ties in every TopK go to the lowest expert index; values are compared as
    numbers (+0 == -0);
  * votes are post-softmax probabilities over all M experts, masked to each
    token's own top-K (model K), not renormalised;
  * only experts nominated by at least one token can enter a vote coreset, so
    the coreset may be smaller than C;
  * a token uses k_eff = min(K, |coreset|) experts; unused slots carry
    index -1 and weight 0;
  * act = "sigmoid": the router weight of an expert is sigmoid(logit); votes add
    these scores and a token's gates are its selected scores divided by their
    sum; rankings still compare logits (the sigmoid is monotone);
  * renorm = True (the alternative reading of how Sec. 4.2 adds up the votes):
    a token's K votes are divided by their sum, so every token casts a total
    weight of one;
  * k_route (Sec. 5.3, the study of the active expert count): the coreset is elected
    with the model's K, then each token uses only its k_route < K best coreset
    experts; gates are normalised over those;
  * cumulative_skip: experts i..k (rank order) are dropped when the sum of their
    gates is below beta times the sum of all k gates (strictly); the largest such
    suffix is taken, the best expert always stays, and the surviving gates are
    re-normalised over the survivors (the normalisation of Eq. 1);
  * group-limited routing (n_group > 1): the M experts form n_group equal groups
    of consecutive indices; a token scores each group by its best router weight
    ("max") or by the sum of its two best ("top2sum"), keeps the topk_group best
    groups (ties to the lowest group index) and never ranks an expert outside
    them: neither in its own top-K that nominates and votes (stage 1) nor in
    its choice inside the coreset (stage 2).  A token whose allowed groups hold
    fewer than k coreset experts uses only those (none: it gets no routed expert);
  * DES-Seq with k_seq == 0 picks the largest k' <= K whose union has at most C
    members; if even k' = 1 overflows, the C most often top-1-nominated experts
    are kept (ties to the lowest index).

Pins: tests/test_oracle_pins.py (brute force over subsets, a hand-worked
3-token x 5-expert example, the closed form for uniform routing, Table 1's
rounding, reductions to a plain numpy MLP and to a dense one-hot einsum,
the skipping rule on hand-computed gates and against enumeration of every cut,
group limits against a scan of the global ranking, an enumeration of pairs and a
hand-worked example, and the invariants the method fixes).  The token-level statistics the paper
reports on trained routers (hit-rate cosine similarity, accuracy) are
"parity unpinned": they need trained weights.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

MODES = ("vanilla", "seq", "vote")


# --------------------------------------------------------------------------
# Router
# --------------------------------------------------------------------------
def router_logits(x: np.ndarray, w_router: np.ndarray,
                  bias: Optional[np.ndarray] = None) -> np.ndarray:
    """Router scores G(x) for every token (Background, definition of G).

    x: [T, D]; w_router: [M, D] (row i is expert i's router vector);
    bias: [M] or None.  Returns float64 [T, M].
    """
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w_router, dtype=np.float64)
    logits = x @ w.T
    if bias is not None:
        logits = logits + np.asarray(bias, dtype=np.float64)[None, :]
    return logits


def softmax_rows(logits: np.ndarray) -> np.ndarray:
    """Per-token softmax over all M experts (Sec. 4.3)."""
    z = np.asarray(logits, dtype=np.float64)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


ACTS = ("softmax", "sigmoid")


def router_scores(logits: np.ndarray, act: str = "softmax") -> np.ndarray:
    """Router weights of every (token, expert): sigma of Sec. 4.1.  softmax over
    the M experts of a token, or the logistic sigmoid of each logit."""
    if act == "softmax":
        return softmax_rows(logits)
    if act == "sigmoid":
        return 1.0 / (1.0 + np.exp(-np.asarray(logits, dtype=np.float64)))
    raise ValueError(f"unknown router activation {act!r}")


def rank_order(row: Sequence[float]) -> List[int]:
    """Expert ids of one token sorted best first: value descending, ties to the
    lowest index (TopK below Eq. 1 with the tie rule stated in the header)."""
    vals = [float(v) for v in row]
    for v in vals:
        if not math.isfinite(v):
            raise ValueError("router logits must be finite")
    return sorted(range(len(vals)), key=lambda i: (-vals[i], i))


def topk(row: Sequence[float], k: int, allowed: Optional[Sequence[bool]] = None) -> List[int]:
    """TopK(row, k) in rank order; with `allowed`, among the allowed experts only."""
    order = rank_order(row)
    if allowed is not None:
        order = [i for i in order if allowed[i]]
    return order[:k]


GROUP_SCORES = ("max", "top2sum")


def group_limited(scores: Sequence[float], n_group: int, topk_group: int,
                  kind: str = "max") -> Tuple[List[bool], float]:
    """Group-limited routing for one token (see the header).  scores: the token's
    M router weights (router_scores).  Returns (allowed [M], margin) where margin
    is the relative gap between the score of the last group kept and of the first
    group left out (inf when every group is kept)."""
    M = len(scores)
    if n_group < 1 or M % n_group != 0:
        raise ValueError("the experts must split into equal groups")
    if not 1 <= topk_group <= n_group:
        raise ValueError("1 <= topk_group <= n_group")
    if kind not in GROUP_SCORES:
        raise ValueError(f"unknown group score {kind!r}")
    size = M // n_group
    gscore = []
    for g in range(n_group):
        members = sorted((float(scores[i]) for i in range(g * size, (g + 1) * size)), reverse=True)
        gscore.append(members[0] if kind == "max" else sum(members[:2]))
    order = sorted(range(n_group), key=lambda g: (-gscore[g], g))
    kept = set(order[:topk_group])
    allowed = [(i // size) in kept for i in range(M)]
    if topk_group < n_group:
        last_in, first_out = gscore[order[topk_group - 1]], gscore[order[topk_group]]
        margin = (last_in - first_out) / abs(last_in) if last_in != 0 else 0.0
    else:
        margin = math.inf
    return allowed, float(margin)


def allowed_experts(logits: np.ndarray, act: str, n_group: int, topk_group: int,
                    kind: str) -> Tuple[Optional[np.ndarray], float]:
    """group_limited for every token of a sequence.  Returns (allowed bool [N, M]
    or None when there is no group limit, smallest margin)."""
    if n_group <= 1:
        return None, math.inf
    P = router_scores(logits, act)
    rows, margin = [], math.inf
    for n in range(P.shape[0]):
        a, m = group_limited(P[n], n_group, topk_group, kind)
        rows.append(a)
        margin = min(margin, m)
    return np.array(rows, dtype=bool), margin


# --------------------------------------------------------------------------
# Coreset selection functions Phi
# --------------------------------------------------------------------------
def _row(allowed: Optional[np.ndarray], n: int):
    return None if allowed is None else allowed[n]


def coreset_seq(logits: np.ndarray, k_seq: int, allowed: Optional[np.ndarray] = None) -> List[int]:
    """Eq. 5 / Alg. 2: union over tokens of each token's top-k_seq experts."""
    core = set()
    for n in range(logits.shape[0]):
        core |= set(topk(logits[n], k_seq, _row(allowed, n)))
    return sorted(core)


def coreset_seq_capped(logits: np.ndarray, K: int, C: int,
                       allowed: Optional[np.ndarray] = None) -> Tuple[List[int], int]:
    """DES-Seq under a size cap C (extension; see header).  Returns
    (coreset ascending, k_seq used); k_seq used is 0 in the overflow case."""
    best_k = 0
    for kp in range(1, K + 1):
        if len(coreset_seq(logits, kp, allowed)) <= C:
            best_k = kp
        else:
            break  # union size is monotone in k'
    if best_k > 0:
        return coreset_seq(logits, best_k, allowed), best_k
    M = logits.shape[1]
    nominations = [0] * M
    for n in range(logits.shape[0]):
        nominations[topk(logits[n], 1, _row(allowed, n))[0]] += 1
    cand = [i for i in range(M) if nominations[i] > 0]
    cand.sort(key=lambda i: (-nominations[i], i))
    return sorted(cand[:C]), 0


def vote_vector(logits: np.ndarray, K: int, act: str = "softmax", renorm: bool = False,
                allowed: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Alg. 3, the masking and the summing step: V_i = sum over tokens of the token's router weight
    for expert i, counted only where i is inside that token's own top-K.
    renorm: each token's K weights are first divided by their sum.
    Returns (V float64 [M], nominated bool [M])."""
    N, M = logits.shape
    P = router_scores(logits, act)
    V = np.zeros(M, dtype=np.float64)
    nominated = np.zeros(M, dtype=bool)
    for n in range(N):
        mine = topk(logits[n], K, _row(allowed, n))
        scale = 1.0 / sum(P[n, i] for i in mine) if renorm else 1.0
        for i in mine:
            V[i] += P[n, i] * scale
            nominated[i] = True
    return V, nominated


def coreset_vote(logits: np.ndarray, K: int, C: int, act: str = "softmax", renorm: bool = False,
                 allowed: Optional[np.ndarray] = None) -> Tuple[List[int], np.ndarray, float]:
    """Eq. 6 / Alg. 3: the C experts with the largest total vote among the
    nominated ones (ties to the lowest index).

    Returns (coreset ascending, V, margin) where margin is the relative gap
    (V_(C) - V_(C+1)) / V_(C) between the last expert taken and the first one
    left out (inf when nothing was left out).
    """
    V, nominated = vote_vector(logits, K, act, renorm, allowed)
    cand = [i for i in range(len(V)) if nominated[i]]
    cand.sort(key=lambda i: (-V[i], i))
    taken = cand[:C]
    if len(cand) > C and len(taken) > 0:
        last_in, first_out = V[taken[-1]], V[cand[C]]
        margin = float((last_in - first_out) / last_in) if last_in > 0 else 0.0
    else:
        margin = math.inf
    return sorted(taken), V, margin


def select_coreset(logits: np.ndarray, mode: str, K: int, C: int,
                   k_seq: int = 0, act: str = "softmax", renorm: bool = False,
                   allowed: Optional[np.ndarray] = None) -> Dict[str, object]:
    """Stage 1 of Alg. 1 for one sequence: coreset = Phi(logits).  allowed
    [N, M]: the experts each token may rank (group-limited routers)."""
    if mode not in MODES:
        raise ValueError(f"unknown mode {mode!r}")
    N, M = logits.shape
    out: Dict[str, object] = {"votes": None, "k_seq_used": 0, "margin": math.inf}
    if mode == "vanilla":
        out["coreset"] = list(range(M))           # Eq. 1: no restriction
    elif mode == "seq":
        if k_seq > 0:
            out["coreset"] = coreset_seq(logits, k_seq, allowed)
            out["k_seq_used"] = k_seq
        else:
            core, used = coreset_seq_capped(logits, K, C, allowed)
            out["coreset"], out["k_seq_used"] = core, used
    else:
        core, V, margin = coreset_vote(logits, K, C, act, renorm, allowed)
        out["coreset"], out["votes"], out["margin"] = core, V, margin
    return out


# --------------------------------------------------------------------------
# Stage 2: constrained routing
# --------------------------------------------------------------------------
def constrained_topk(row: Sequence[float], coreset: Sequence[int], K: int,
                     allowed: Optional[Sequence[bool]] = None) -> List[int]:
    """Alg. 1 stage 2: S_n = TopK(row restricted to the coreset, K), rank order.
    allowed: the experts this token may rank at all (group-limited routers)."""
    inside = set(int(c) for c in coreset)
    return [i for i in rank_order(row) if i in inside and (allowed is None or allowed[i])][:K]


def gates(row: Sequence[float], selected: Sequence[int], act: str = "softmax") -> np.ndarray:
    """Alg. 1 stage 2: g_n = the token's router weights over S_n divided by their
    sum (the normalisation of Eq. 1).  For the softmax router that is the
    softmax of the selected logits, P_i / sum_{j in S_n} P_j."""
    if len(selected) == 0:
        return np.zeros(0, dtype=np.float64)
    z = np.array([float(row[i]) for i in selected], dtype=np.float64)
    if act == "sigmoid":
        e = 1.0 / (1.0 + np.exp(-z))
    elif act == "softmax":
        e = np.exp(z - z.max())
    else:
        raise ValueError(f"unknown router activation {act!r}")
    return e / e.sum()


def cumulative_skip(g: np.ndarray, beta: float) -> Tuple[int, float]:
    """Sec. 5.1 (Baselines), the adapted NAEE rule on one token's gates g (rank
    order, best first): skip experts i..k when sum_{u=i..k} g_u < beta * sum_u g_u.
    Returns (number of experts kept, margin), margin = the smallest relative
    distance |suffix - beta * total| / total over all cuts (how close the
    decision came to flipping)."""
    g = np.asarray(g, dtype=np.float64)
    k = len(g)
    if k == 0 or beta <= 0.0:
        return k, math.inf
    total = float(g.sum())
    keep, margin = k, math.inf
    suffix = 0.0
    for i in range(k - 1, 0, -1):          # the best expert (i = 0) is never skipped
        suffix += float(g[i])
        margin = min(margin, abs(suffix - beta * total) / total)
        if suffix < beta * total:
            keep = i
    return keep, margin


# --------------------------------------------------------------------------
# Experts
# --------------------------------------------------------------------------
def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def expert_ffn(x: np.ndarray, wg: np.ndarray, wu: np.ndarray, wd: np.ndarray) -> np.ndarray:
    """E(x) for one token.  wg, wu: [F, D] (row f is the weight vector of
    intermediate unit f); wd: [D, F] (row d produces output coordinate d).
    E(x) = wd @ (silu(wg @ x) * (wu @ x))."""
    h = silu(wg @ x) * (wu @ x)
    return wd @ h


class _F64Cache:
    """Memo of float64 upcasts of per-expert weight matrices (conversion only)."""

    def __init__(self, w_gate, w_up, w_down):
        self.w = (w_gate, w_up, w_down)
        self.memo: Dict[int, Tuple[np.ndarray, np.ndarray, np.ndarray]] = {}

    def get(self, e: int):
        if e not in self.memo:
            self.memo[e] = tuple(np.asarray(m[e], dtype=np.float64) for m in self.w)
        return self.memo[e]


# --------------------------------------------------------------------------
# The layer (Alg. 1)
# --------------------------------------------------------------------------
def route_block(logits: np.ndarray, mode: str, K: int, C: int, k_seq: int = 0,
                k_route: int = 0, skip_beta: float = 0.0, act: str = "softmax",
                renorm: bool = False, n_group: int = 0, topk_group: int = 0,
                group_score: str = "max") -> Dict[str, object]:
    """Routing part of Alg. 1 for ONE sequence given its logits [N, M]:
    coreset, per-token S_n (rank order, padded with -1) and gates (padded 0).
    k_route > 0: a token uses only its k_route best coreset experts (the
    election still uses K).  skip_beta > 0: cumulative_skip on every token.
    act, renorm: router activation and vote normalisation; n_group, topk_group,
    group_score: group-limited routing (see the header)."""
    logits = np.asarray(logits, dtype=np.float64)
    N, M = logits.shape
    allowed, group_margin = allowed_experts(logits, act, n_group, topk_group, group_score)
    sel = select_coreset(logits, mode, K, C, k_seq, act, renorm, allowed)
    core = sel["coreset"]
    idx = -np.ones((N, K), dtype=np.int32)
    w = np.zeros((N, K), dtype=np.float64)
    skip_margin = math.inf
    for n in range(N):
        s_n = constrained_topk(logits[n], core, k_route if k_route > 0 else K, _row(allowed, n))
        g_n = gates(logits[n], s_n, act)
        if skip_beta > 0.0:
            keep, m = cumulative_skip(g_n, skip_beta)
            skip_margin = min(skip_margin, m)
            s_n = s_n[:keep]
            g_n = gates(logits[n], s_n, act)
        idx[n, :len(s_n)] = s_n
        w[n, :len(s_n)] = g_n
    sel.update(topk_idx=idx, topk_w=w, skip_margin=skip_margin, group_margin=group_margin)
    return sel


def moe_forward(x: np.ndarray, w_router: np.ndarray, bias: Optional[np.ndarray],
                w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray,
                K: int, C: int, mode: str, k_seq: int = 0,
                shared: Optional[Tuple[np.ndarray, np.ndarray, np.ndarray]] = None,
                logits_override: Optional[np.ndarray] = None,
                compute_y: bool = True, residual: bool = False,
                only_tokens: Optional[Sequence[Tuple[int, int]]] = None,
                k_route: int = 0, skip_beta: float = 0.0, act: str = "softmax",
                renorm: bool = False, n_group: int = 0, topk_group: int = 0,
                group_score: str = "max") -> Dict[str, object]:
    """Alg. 1 for B independent sequences.

    x: [B, N, D].  w_router [M, D]; w_gate, w_up [M, F, D]; w_down [M, D, F].
    shared: optional (wg [Fs, D], wu [Fs, D], wd [D, Fs]) always-on expert added
    with weight 1.  logits_override [B, N, M]: use these router logits instead
    of computing them (the routing decisions are then a function of exactly
    these numbers).  Each sequence elects its own coreset.  only_tokens: compute
    y only for these (sequence, token) pairs (the rest of y stays NaN); routing
    is always computed for every token.  k_route, skip_beta, act, renorm,
    n_group, topk_group, group_score: see route_block.
    """
    x = np.asarray(x)
    B, N, D = x.shape
    M = w_router.shape[0]
    x64 = x.astype(np.float64)
    if logits_override is not None:
        logits = np.asarray(logits_override, dtype=np.float64).reshape(B, N, M)
    else:
        logits = router_logits(x64.reshape(B * N, D), w_router, bias).reshape(B, N, M)

    topk_idx = -np.ones((B, N, K), dtype=np.int32)
    topk_w = np.zeros((B, N, K), dtype=np.float64)
    coresets: List[List[int]] = []
    votes: List[Optional[np.ndarray]] = []
    margins: List[float] = []
    k_seq_used: List[int] = []
    skip_margin = group_margin = math.inf
    for b in range(B):
        r = route_block(logits[b], mode, K, C, k_seq, k_route, skip_beta, act, renorm,
                        n_group, topk_group, group_score)
        skip_margin = min(skip_margin, r["skip_margin"])
        group_margin = min(group_margin, r["group_margin"])
        topk_idx[b], topk_w[b] = r["topk_idx"], r["topk_w"]
        coresets.append(r["coreset"])
        votes.append(r["votes"])
        margins.append(r["margin"])
        k_seq_used.append(r["k_seq_used"])

    counts = np.zeros(M, dtype=np.int32)        # cnt_i of Eq. 2, summed over sequences
    for e in topk_idx.reshape(-1):
        if e >= 0:
            counts[e] += 1
    n_unique = int((counts > 0).sum())           # |union_n S_n|

    y = None
    if compute_y:
        cache = _F64Cache(w_gate, w_up, w_down)
        y = np.zeros((B, N, D), dtype=np.float64)
        wanted = None
        if only_tokens is not None:
            y[:] = np.nan
            wanted = set((int(b), int(n)) for b, n in only_tokens)
        sh = None
        if shared is not None:
            sh = tuple(np.asarray(m, dtype=np.float64) for m in shared)
        for b in range(B):
            for n in range(N):
                if wanted is not None and (b, n) not in wanted:
                    continue
                acc = np.zeros(D, dtype=np.float64)
                for j in range(K):
                    e = int(topk_idx[b, n, j])
                    if e < 0:
                        continue
                    wg, wu, wd = cache.get(e)
                    acc += topk_w[b, n, j] * expert_ffn(x64[b, n], wg, wu, wd)
                if sh is not None:
                    acc += expert_ffn(x64[b, n], *sh)
                if residual:
                    acc += x64[b, n]
                y[b, n] = acc
    return dict(logits=logits, topk_idx=topk_idx, topk_w=topk_w, counts=counts,
                n_unique=n_unique, coresets=coresets, votes=votes, margins=margins,
                k_seq_used=k_seq_used, y=y, skip_margin=skip_margin, group_margin=group_margin)


def moe_stack_forward(x: np.ndarray, layers: Sequence[dict], K: int, C: int, mode: str,
                      k_seq: int = 0) -> Tuple[np.ndarray, List[Dict[str, object]]]:
    """x_{l+1} = x_l + MoE_l(x_l) for a list of layers (each a dict with
    w_router, bias, w_gate, w_up, w_down and optionally shared)."""
    cur = np.asarray(x, dtype=np.float64)
    per_layer = []
    for lw in layers:
        r = moe_forward(cur, lw["w_router"], lw.get("bias"), lw["w_gate"], lw["w_up"],
                        lw["w_down"], K, C, mode, k_seq, shared=lw.get("shared"),
                        residual=True)
        per_layer.append(r)
        cur = r["y"]
    return cur, per_layer


# --------------------------------------------------------------------------
# Attention around the MoE layers (the wider decoding step)
# --------------------------------------------------------------------------
def block_attention(x: np.ndarray, wq: np.ndarray, wk: np.ndarray, wv: np.ndarray, wo: np.ndarray,
                    k_cache: np.ndarray, v_cache: np.ndarray, n_heads: int, n_kv_heads: int,
                    residual: bool = False) -> np.ndarray:
    """The attention sub-layer of one decoding step of a block-parallel decoder with
    cached context (Sec. 5.1: a block of N tokens, cached prefix and suffix positions).
    The paper treats attention as a fixed, non-MoE cost (Fig. 2 left, Sec. 5.2) and
    does not define it; this is plain multi-head scaled-dot-product attention, every
    block token attending to every cached position and to every token of its own block
    (no causal mask: all block tokens are decoded together), no positional encoding,
    no bias (readings listed in the design notes).

      x        [B, N, D]        hidden states of the block
      wq       [H*dh, D]        row r produces query coordinate r   (likewise wk, wv: [Hkv*dh, D])
      wo       [D, H*dh]        row d produces output coordinate d
      k_cache, v_cache  [B, Hkv, P, dh]   keys / values of the P cached positions
      q = wq x, k = wk x, v = wv x for the block's own tokens; head h of the H query heads
      reads key/value head h // (H / Hkv); for token n and head h
        s_j = <q_n, key_j> / sqrt(dh) over the P cached and the N block keys,
        p = softmax(s),  o_n = sum_j p_j value_j;   y_n = wo [o_n over heads] (+ x_n).
    Everything in float64.  Returns y [B, N, D]."""
    x = np.asarray(x, dtype=np.float64)
    B, N, D = x.shape
    wq, wk, wv, wo = (np.asarray(m, dtype=np.float64) for m in (wq, wk, wv, wo))
    kc = np.asarray(k_cache, dtype=np.float64)
    vc = np.asarray(v_cache, dtype=np.float64)
    H, Hkv = n_heads, n_kv_heads
    dh = wq.shape[0] // H
    assert wq.shape == (H * dh, D) and wk.shape == (Hkv * dh, D) and wv.shape == (Hkv * dh, D)
    assert wo.shape == (D, H * dh) and H % Hkv == 0
    P = kc.shape[2]
    assert kc.shape == (B, Hkv, P, dh) and vc.shape == (B, Hkv, P, dh)
    y = np.zeros((B, N, D), dtype=np.float64)
    for b in range(B):
        q = x[b] @ wq.T                      # [N, H*dh]
        k = x[b] @ wk.T                      # [N, Hkv*dh]
        v = x[b] @ wv.T
        heads = np.zeros((N, H * dh), dtype=np.float64)
        for h in range(H):
            g = h // (H // Hkv)
            keys = np.concatenate([kc[b, g], k[:, g * dh:(g + 1) * dh]], axis=0)   # [P + N, dh]
            vals = np.concatenate([vc[b, g], v[:, g * dh:(g + 1) * dh]], axis=0)
            for n in range(N):
                s = keys @ q[n, h * dh:(h + 1) * dh] / math.sqrt(dh)
                p = np.exp(s - s.max())
                p /= p.sum()
                heads[n, h * dh:(h + 1) * dh] = p @ vals
        y[b] = heads @ wo.T
    return y + x if residual else y


def decoder_stack_forward(x: np.ndarray, layers: Sequence[dict], K: int, C: int, mode: str,
                          n_heads: int, n_kv_heads: int) -> Tuple[np.ndarray, List[Dict[str, object]]]:
    """A stack of decoder layers, each an attention sub-layer followed by a MoE sub-layer,
    both with a residual connection:  a = x + Attn_l(x);  x' = a + MoE_l(a).  Each layer is
    a dict with wq, wk, wv, wo, k_cache, v_cache and the MoE tensors of moe_stack_forward.
    Returns the final hidden states and the per-layer MoE results."""
    cur = np.asarray(x, dtype=np.float64)
    per_layer = []
    for lw in layers:
        a = block_attention(cur, lw["wq"], lw["wk"], lw["wv"], lw["wo"], lw["k_cache"], lw["v_cache"],
                            n_heads, n_kv_heads, residual=True)
        r = moe_forward(a, lw["w_router"], lw.get("bias"), lw["w_gate"], lw["w_up"], lw["w_down"],
                        K, C, mode, shared=lw.get("shared"), residual=True)
        per_layer.append(r)
        cur = r["y"]
    return cur, per_layer


# --------------------------------------------------------------------------
# Closed forms the paper prints
# --------------------------------------------------------------------------
def expected_unique_uniform(M: int, K: int, N: int) -> float:
    """Sec. 3: expected |union S_n| under uniform routing, M (1 - (1 - K/M)^N)."""
    return M * (1.0 - (1.0 - K / M) ** N)


def coreset_size_from_beta(beta: float, M: int) -> int:
    """M_core = beta * M (Sec. 5.1); Table 1's printed sizes fix the rounding
    to floor (0.15*256 -> 38, 0.10*256 -> 25, 0.6*64 -> 38, 0.4*64 -> 25).
    The product is formed exactly (decimal beta) so 0.15*256 is 38.4, not
    38.39999..."""
    from fractions import Fraction
    return int(math.floor(Fraction(str(beta)) * M))
