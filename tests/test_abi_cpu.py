"""Host-side checks of the C-ABI library: it loads, exports every symbol the
header declares, sizes its workspace and rejects bad arguments before any
launch.  No compute call is made, so this runs without a GPU."""
import ctypes
import os
import re

import pytest

from paper_2602_00879_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "des.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(des_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS), (names, B.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def _shape(**kw):
    base = dict(n_seqs=1, n_tokens=32, hidden=2048, n_experts=128, ffn=768, top_k=8, coreset=32,
                mode="vote", dtype="bf16")
    base.update(kw)
    return B.make_shape(**base)


def test_workspace_and_capacity_are_host_only():
    s = _shape()
    assert B.des_coreset_capacity(s) == 32
    assert B.des_coreset_capacity(_shape(mode="vanilla")) == 128
    assert B.des_coreset_capacity(_shape(coreset=500)) == 128
    n = B.des_workspace_bytes(s)
    TK = 32 * 8
    assert n >= TK * 768 * 2 + TK * 2048 * 4 and n % 256 == 0
    assert B.des_workspace_bytes(_shape(ffn_shared=512)) > n
    assert B.des_stack_workspace_bytes(s) > n


@pytest.mark.parametrize("kw,code", [
    (dict(mode=7), -3),
    (dict(dtype=5), -4),
    (dict(dtype="f32", weight_layout=1), -4),
    (dict(n_tokens=0), -2),
    (dict(top_k=129), -2),
    (dict(top_k=33, n_experts=64), -2),
    (dict(n_experts=513), -2),
    (dict(coreset=0), -2),
    (dict(k_seq=9), -2),
    (dict(hidden=2040), -2),
    (dict(ffn=100), -2),
    (dict(n_seqs=200), -2),
    (dict(mode="seq", k_seq=2, coreset=32), -2),   # union of 32*2 may not fit 32
    (dict(residual=2), -2),
    (dict(k_route=9), -2),
    (dict(k_route=-1), -2),
    (dict(skip_beta=1.0), -2),
    (dict(skip_beta=-0.1), -2),
    (dict(skip_beta=float("nan")), -2),
    (dict(router_act=2), -3),
    (dict(vote_renorm=2), -2),
    (dict(vote_atomic=2), -2),
    (dict(n_group=-1), -2),
    (dict(n_group=3, topk_group=1), -2),                 # 128 experts do not split into 3 groups
    (dict(n_group=32, topk_group=4), -2),                # groups of 4 experts: not whole lanes
    (dict(n_group=8, topk_group=0), -2),
    (dict(n_group=8, topk_group=9), -2),
    (dict(n_group=16, topk_group=1, top_k=9), -2),       # 8 allowed experts cannot fill K = 9
    (dict(n_group=8, topk_group=4, group_score=0), -3),
    (dict(n_group=8, topk_group=4, group_score=3), -3),
])
def test_bad_shapes_are_rejected_before_launch(kw, code):
    s = _shape(**kw)
    L = B.lib()
    args = [ctypes.c_void_p(256 * (i + 1)) for i in range(18)]  # never dereferenced
    rc = L.des_moe_forward(ctypes.byref(s), *args, ctypes.c_size_t(1 << 40), None)
    assert rc == code, B.strerror(rc)
    assert B.des_workspace_bytes(s) == 0


def test_null_and_workspace_errors():
    s = _shape()
    L = B.lib()
    one = ctypes.c_void_p(256)
    args = [ctypes.c_void_p(256 * (i + 1)) for i in range(18)]   # never dereferenced
    assert L.des_moe_forward(ctypes.byref(s), *args, ctypes.c_size_t(16), None) == -5
    misaligned = list(args)
    misaligned[17] = ctypes.c_void_p(257 + 3)
    assert L.des_moe_forward(ctypes.byref(s), *misaligned, ctypes.c_size_t(1 << 40), None) == -5
    bad = list(args)
    bad[0] = None
    assert L.des_moe_forward(ctypes.byref(s), *bad, ctypes.c_size_t(1 << 40), None) == -1
    sh = _shape(ffn_shared=512)
    no_shared = list(args)
    no_shared[6] = None
    assert L.des_moe_forward(ctypes.byref(sh), *no_shared, ctypes.c_size_t(1 << 40), None) == -1
    assert L.des_route(ctypes.byref(s), None, one, None, one, None, None) == -1
    assert L.des_select_coreset(ctypes.byref(s), one, None, one, None, None, None) == -1
    assert L.des_pack_expert_weights(one, one, 1, 16, 32, None) == -2
    assert L.des_pack_expert_weights(one, ctypes.c_void_p(512), 1, 15, 32, None) == -2
    assert L.des_moe_forward(None, *args, ctypes.c_size_t(0), None) == -1
    assert "workspace" in B.strerror(-5) and B.strerror(0) == "ok"
    # x and y must differ
    alias = list(args)
    alias[9] = alias[0]
    assert L.des_moe_forward(ctypes.byref(s), *alias, ctypes.c_size_t(1 << 40), None) == -2


def test_stack_entry_points_reject_aliased_input_and_output():
    s = _shape(residual=1)
    L = B.lib()
    L.des_moe_stack_forward.restype = ctypes.c_int
    ptrs = [ctypes.c_void_p(256 * (i + 1)) for i in range(14)]   # never dereferenced
    # (shape, n_layers, x, w_router, bias, wg, wu, wd, sg, su, sd, y, counts, n_unique, workspace, bytes, stream)
    args = list(ptrs)
    args[9] = args[0]                                            # y = x
    rc = L.des_moe_stack_forward(ctypes.byref(s), 1, *args[:13], ctypes.c_size_t(1 << 40), None)
    assert rc == -2
    ok = B.make_attn_shape(32, 4, 128, 16, 16)
    d = [ctypes.c_void_p(256 * (i + 1)) for i in range(19)]
    d[15] = d[0]                                                 # y = x
    assert L.des_decoder_stack_forward(ctypes.byref(s), ctypes.byref(ok), 1, *d, ctypes.c_size_t(1 << 40), None) == -2


def test_attention_shapes_are_checked_on_the_host():
    s = _shape()
    ok = B.make_attn_shape(32, 4, 128, 16, 16)
    n = B.des_attention_workspace_bytes(s, ok)
    T = 32
    assert n >= T * (32 * 128 * 2 + 2 * 4 * 128) * 2 and n % 256 == 0
    assert B.des_decoder_workspace_bytes(s, ok) >= n + B.des_stack_workspace_bytes(s)
    for bad in (B.make_attn_shape(32, 5, 128, 16, 16),     # heads do not split into groups
                B.make_attn_shape(32, 4, 100, 16, 16),     # head_dim not a multiple of 8
                B.make_attn_shape(3, 3, 8, 0, 0),          # H * dh not a multiple of 128
                B.make_attn_shape(32, 4, 128, -1, 0),
                B.make_attn_shape(32, 4, 128, 4000, 200),  # window beyond the limit
                B.make_attn_shape(16, 16, 256, 16, 16),    # head_dim beyond 128
                B.make_attn_shape(32, 4, 128, 600, 200)):  # one head's window exceeds LDS
        assert B.des_attention_workspace_bytes(s, bad) == 0
        assert B.des_decoder_workspace_bytes(s, bad) == 0
    assert B.des_attention_workspace_bytes(_shape(dtype="f32"), ok) == 0
    L = B.lib()
    a = [ctypes.c_void_p(256 * (i + 1)) for i in range(9)]      # never dereferenced
    call = lambda sh, at, args, nbytes: L.des_block_attention(ctypes.byref(sh), ctypes.byref(at), *args,
                                                              ctypes.c_size_t(nbytes), None)
    assert call(_shape(dtype="f32"), ok, a, 1 << 40) == -4
    assert call(s, ok, a, 16) == -5
    no_cache = list(a)
    no_cache[5] = None
    assert call(s, ok, no_cache, 1 << 40) == -1
    alias = list(a)
    alias[7] = alias[0]
    assert call(s, ok, alias, 1 << 40) == -2
    d = [ctypes.c_void_p(256 * (i + 1)) for i in range(19)]
    assert L.des_decoder_stack_forward(ctypes.byref(s), ctypes.byref(ok), 0, *d, ctypes.c_size_t(1 << 40), None) == -2
    assert L.des_decoder_stack_forward(ctypes.byref(s), ctypes.byref(ok), 2, *d, ctypes.c_size_t(16), None) == -5
    d[0] = None
    assert L.des_decoder_stack_forward(ctypes.byref(s), ctypes.byref(ok), 2, *d, ctypes.c_size_t(1 << 40), None) == -1


def test_coreset_from_beta_matches_table_1_rounding():
    """M_core = floor(beta * M): the sizes printed in Table 1 of the paper, and the
    oracle's exact-fraction version on a grid of decimal budgets."""
    from oracle import des_oracle as O
    assert B.des_coreset_from_beta(0.15, 256) == 38 and B.des_coreset_from_beta(0.10, 256) == 25
    assert B.des_coreset_from_beta(0.6, 64) == 38 and B.des_coreset_from_beta(0.4, 64) == 25
    for M in (8, 10, 64, 100, 128, 256, 512):
        for pct in range(1, 101):
            beta = pct / 100.0
            assert B.des_coreset_from_beta(beta, M) == max(1, O.coreset_size_from_beta(beta, M)), (beta, M)
    assert B.des_coreset_from_beta(0.0, 64) == 0 and B.des_coreset_from_beta(1.5, 64) == 0
    assert B.des_coreset_from_beta(0.5, 0) == 0
