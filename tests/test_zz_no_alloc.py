"""des_moe_forward_builtin_ws - the entry point for callers that cannot allocate -
against des_moe_forward on the same inputs: two calls in a row on the library's
built-in scratch, the second on a smaller block (what the first left behind in the
scratch must not matter), outputs bit-identical to the caller-workspace entry point and
within the usual tolerances of the CPU oracle."""
import ctypes

import pytest
import torch

from paper_2602_00879_amd import binding as B
from paper_2602_00879_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _both(cfg, mode, layout_packed):
    layer = W.make_layer(cfg)
    dev = H.layer_to_device(layer)
    wg, wu, wd, sh = dev["w_gate"], dev["w_up"], dev["w_down"], dev["shared"]
    layout = B.DES_LAYOUT_ROWMAJOR
    if layout_packed:
        wg, wu, wd = (B.des_pack_expert_weights(t) for t in (wg, wu, wd))
        sh = tuple(B.des_pack_expert_weights(m) for m in sh) if sh else None
        layout = B.DES_LAYOUT_PACKED
    shape = H.shape_of(cfg, mode, layout=layout)
    print(f"no-alloc {cfg.name} N={cfg.n_tokens} {mode} packed={layout_packed}", flush=True)
    ref = B.des_moe_forward(shape, dev["x"], dev["w_router"], dev["bias"], wg, wu, wd, shared=sh)
    torch.cuda.synchronize()
    outs = B.MoeBuffers(shape, "cuda", torch.bfloat16, with_workspace=False)
    before = torch.cuda.memory_allocated()
    got = B.des_moe_forward_builtin_ws(shape, dev["x"], dev["w_router"], dev["bias"], wg, wu, wd,
                                       shared=sh, buffers=outs)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for name in ("y", "logits", "topk_idx", "topk_w", "expert_counts", "n_unique", "coreset_idx",
                 "coreset_size"):
        assert torch.equal(getattr(got, name), getattr(ref, name)), name
    H.check_against_oracle(cfg, layer, got, mode, label=f"no-alloc {cfg.name}")


def test_builtin_scratch_matches_caller_workspace():
    big = W.CONFIGS["m256_shared"].with_(n_experts=64, ffn=256, ffn_shared=256, hidden=512, name="na_big")
    _both(big.with_(n_tokens=80), "vote", True)       # long-block kernels, shared expert
    _both(big.with_(n_tokens=24, seed=77), "vote", True)   # then a smaller block on the same scratch
    _both(big.with_(n_tokens=7, seed=78), "seq", False)


def test_builtin_scratch_refuses_what_does_not_fit():
    cfg = W.CONFIGS["stack48"]  # 256 token rows: about 20 MB of scratch
    shape = H.shape_of(cfg, "vote")
    assert B.des_workspace_bytes(shape) > B.BUILTIN_WORKSPACE_BYTES
    args = [ctypes.c_void_p(256 * (i + 1)) for i in range(17)]  # never dereferenced
    rc = B.lib().des_moe_forward_builtin_ws(ctypes.byref(shape), *args, None)
    assert rc == -5 and "built-in" in B.strerror(rc)
