"""ded_tree_attention_static (the entry point that allocates nothing: its transient buffers live in the library's
own device array) against ded_tree_attention (the same buffers in the caller's workspace), through the C ABI.
Both run the same kernels with the same key-range split, so the outputs must be equal bit for bit; the oracle
bounds the error of both.  Two calls in a row, the second on a smaller input, then a call that does not fit."""
import numpy as np
import pytest

import ded_inputs as di
import oracle

pytestmark = pytest.mark.gpu


def _inputs(ver, H, Hkv, P, N, max_nodes, seed):
    from paper_2407_12021_amd.binding import _to_device
    import torch
    x = di.attention_inputs(H, Hkv, 128, P, N, seed=seed)
    pad = lambda a, axis: np.concatenate(
        [a, np.zeros(a.shape[:axis] + (max_nodes - N,) + a.shape[axis + 1:], a.dtype)], axis=axis)
    q = _to_device(pad(x["q"], 0), ver.device, "bf16")[None]
    kt = _to_device(pad(x["k_tree"], 1), ver.device, "bf16")[None]
    vt = _to_device(pad(x["v_tree"], 1), ver.device, "bf16")[None]
    return x, q, kt, vt, torch


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch
    assert torch.cuda.is_available()
    from paper_2407_12021_amd import Verifier
    from paper_2407_12021_amd import binding as B
    assert B.ded_static_scratch_bytes() == 32 << 20
    H, Hkv, max_nodes = 32, 8, 64
    cfg = di.ModelConfig("attn-static", 1, 128, H, Hkv, 128, 128, 16)
    ver = Verifier(cfg, di.make_weights(cfg, seed=0), max_batch=1, kv_capacity=2048 + max_nodes, max_nodes=max_nodes)
    for P, N, seed in ((2000, 64, 11), (333, 20, 12)):  # the second call is smaller: stale scratch must not matter
        x, q, kt, vt, _ = _inputs(ver, H, Hkv, P, N, max_nodes, seed)
        parent = di.random_tree(N, None, seed=seed)
        ver.kv_store(0, 0, 0, x["k_prefix"], x["v_prefix"])
        out_s = torch.zeros_like(q)
        ver.tree_attention(0, [P], [parent], q, kt, vt, out=out_s, static=True)
        out_w = ver.tree_attention(0, [P], [parent], q, kt, vt)
        torch.cuda.synchronize()
        assert torch.equal(out_s, out_w), (P, N)
        got = out_s[0, :N].float().cpu().numpy()
        kk = np.concatenate([oracle.widen(x["k_prefix"]), oracle.widen(x["k_tree"])], axis=1).transpose(1, 0, 2)
        vv = np.concatenate([oracle.widen(x["v_prefix"]), oracle.widen(x["v_tree"])], axis=1).transpose(1, 0, 2)
        vis = np.concatenate([np.ones((N, P), bool), oracle.ancestor_mask(parent)], axis=1)
        ref = oracle.masked_attention(oracle.widen(x["q"]), kk, vv, vis)
        err = np.abs(got - ref).max()
        print(f"static attention, prefix {P}, {N} nodes: max |o error| {err:.3e}")
        assert err <= 8e-3, err  # bf16 output: the bound of the attention-only parity test
    ver.close()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    assert torch.cuda.is_available()
    from paper_2407_12021_amd import Verifier
    from paper_2407_12021_amd import binding as B
    H, Hkv, max_nodes, batch, P = 32, 32, 256, 4, 512
    cfg = di.ModelConfig("attn-static-big", 1, 128, H, Hkv, 128, 128, 16)
    ver = Verifier(cfg, di.make_weights(cfg, seed=0), max_batch=batch, kv_capacity=P + max_nodes, max_nodes=max_nodes)
    q = torch.zeros((batch, max_nodes, H, 128), dtype=torch.bfloat16, device=ver.device)
    kt = torch.zeros((batch, Hkv, max_nodes, 128), dtype=torch.bfloat16, device=ver.device)
    out = torch.zeros_like(q)
    parents = [di.chain_tree(max_nodes)] * batch
    # 4 x 256 rows x 4096 features: the re-laid-out queries and output alone are 2 x 16 MiB
    with pytest.raises(B.DedError) as e:
        ver.tree_attention(0, [P] * batch, parents, q, kt, kt, out=out, static=True)
    assert e.value.code == B.DED_ECAP
    # the refusal enqueued nothing and left the context usable: one sequence fits
    out1 = torch.zeros_like(q[:1])
    ver.tree_attention(0, [P], parents[:1], q[:1], kt[:1], kt[:1], out=out1, static=True)
    out2 = ver.tree_attention(0, [P], parents[:1], q[:1], kt[:1], kt[:1])
    torch.cuda.synchronize()
    assert torch.equal(out1, out2)
    ver.close()
