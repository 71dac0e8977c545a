"""Host-only checks of the C ABI: the library loads, exports what the header declares, and the
argument validation (which runs before any launch) returns the documented codes.  No GPU calls."""
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def b():
    from paper_2407_12021_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2407_12021_amd.build import build_library
        build_library()
    return binding


def test_every_declared_symbol_is_exported(b):
    header = open(os.path.join(ROOT, "include", "ded_verify.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ded_[a-z_0-9]+)\s*\(", header))
    assert {"ded_verify_init", "ded_verify_step", "ded_accept"} <= declared
    L = b.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(b.EXPORTS)


def _cfg(b, **kw):
    base = dict(n_layers=2, d_model=256, n_heads=4, n_kv_heads=4, head_dim=64, d_ffn=688, vocab=4096,
                rope_base=10000.0, rms_eps=1e-5, dtype="fp32", max_batch=2, kv_capacity=144, max_nodes=16)
    base.update(kw)
    return b.make_config(**base)


def test_config_validation_and_sizes(b):
    assert b.ded_workspace_bytes(_cfg(b)) > 0
    assert b.ded_kv_layer_bytes(_cfg(b)) == 2 * 4 * 144 * 64 * 4
    for bad in (dict(n_heads=3, n_kv_heads=2), dict(max_nodes=257), dict(head_dim=63), dict(dtype=7),
                dict(dtype="bf16"), dict(vocab=0), dict(rope_base=0.0), dict(max_batch=0)):
        assert b.ded_workspace_bytes(_cfg(b, **bad)) == 0, bad
    ok16 = dict(dtype="bf16", head_dim=128, d_model=256, d_ffn=384, vocab=4096, kv_capacity=192)
    assert b.ded_workspace_bytes(_cfg(b, **ok16)) > 0
    assert b.ded_kv_layer_bytes(_cfg(b, **ok16)) == 2 * 4 * 192 * 128 * 2
    for bad in (dict(kv_capacity=100), dict(d_ffn=400), dict(vocab=4100), dict(d_model=192)):
        assert b.ded_workspace_bytes(_cfg(b, **{**ok16, **bad})) == 0, bad


def test_step_validation_codes(b):
    cfg = _cfg(b)
    par = np.full((2, 16), -1, np.int32)
    tok = np.zeros((2, 16), np.int32)
    par[:, 1:4] = [0, 0, 1]
    V = b.ded_validate_tree
    assert V(cfg, [10, 20], [4, 4], par, tok) == b.DED_OK
    assert V(cfg, [10], [1], par[:1], tok[:1]) == b.DED_OK
    assert V(cfg, [10, 20, 30], [4, 4, 4], np.tile(par[:1], (3, 1)), np.tile(tok[:1], (3, 1))) == b.DED_EINVAL
    assert V(cfg, [10, 20], [0, 4], par, tok) == b.DED_EINVAL
    assert V(cfg, [10, 20], [17, 4], par, tok) == b.DED_EINVAL
    assert V(cfg, [-1, 20], [4, 4], par, tok) == b.DED_EINVAL
    assert V(cfg, [141, 20], [4, 4], par, tok) == b.DED_ECAP
    assert V(cfg, [140, 20], [4, 4], par, tok) == b.DED_OK
    assert V(cfg, [10, 20], [4, 4], None, tok) == b.DED_EINVAL
    bad = par.copy(); bad[1, 0] = 0
    assert V(cfg, [10, 20], [4, 4], bad, tok) == b.DED_ETREE
    bad = par.copy(); bad[0, 2] = 2
    assert V(cfg, [10, 20], [4, 4], bad, tok) == b.DED_ETREE
    bad = par.copy(); bad[0, 3] = -1
    assert V(cfg, [10, 20], [4, 4], bad, tok) == b.DED_ETREE
    bad = par.copy(); bad[0, 9] = 55  # beyond n_nodes: ignored
    assert V(cfg, [10, 20], [4, 4], bad, tok) == b.DED_OK
    t = tok.copy(); t[1, 3] = 4096
    assert V(cfg, [10, 20], [4, 4], par, t) == b.DED_ETOKEN
    t = tok.copy(); t[1, 3] = -5
    assert V(cfg, [10, 20], [4, 4], par, t) == b.DED_ETOKEN


def test_init_rejects_bad_arguments_before_touching_the_device(b):
    with pytest.raises(b.DedError) as e:
        b.ded_verify_init(_cfg(b, max_nodes=300), None, None, 0, 0, None)
    assert e.value.code == b.DED_EINVAL
    with pytest.raises(b.DedError) as e:
        b.ded_verify_init(_cfg(b), None, None, 0, 0, None)
    assert e.value.code == b.DED_EINVAL
    assert b.lib().ded_accept(None, 0, None, None, None, None) == b.DED_EINVAL
    assert b.lib().ded_verify_step(None, 1, None, None, None, None, None) == b.DED_EINVAL
    assert "tree" in b.ded_strerror(b.DED_ETREE)
    assert "NaN" in b.ded_strerror(b.DED_ENONFINITE) and b.DED_ENONFINITE == -8
    assert b.ded_strerror(-99) == "unknown error"


# ---------------------------------------------------------------------------------------------
# ded_build_tree (host only): the pseudo-sequence builder against the oracle, bit-exact
# ---------------------------------------------------------------------------------------------


def test_build_tree_matches_oracle_bit_exact():
    import numpy as np
    import oracle
    from paper_2407_12021_amd import binding as B
    g = np.random.default_rng(21)
    for trial in range(300):
        n_c = int(g.integers(0, 30))
        vocab = int(g.choice([2, 3, 50, 32000]))
        cands = [list(map(int, g.integers(0, vocab, size=int(g.integers(0, 7))))) for _ in range(n_c)]
        budget = int(g.choice([1, 2, 5, 16, 64, 256]))
        rc, parent, token, end = B.ded_build_tree(9, cands, budget)
        assert rc == B.DED_OK
        ref = oracle.build_trie(9, cands, budget)
        assert (parent.tolist(), token.tolist(), end.tolist()) == ref


def test_build_tree_paper_shape_and_validation():
    """24 candidates of length 4 (the paper's n and l, Detailed Experimental Settings): the tree fits the
    97-node budget, is a valid input of the verification step, and every candidate is one of its paths."""
    import numpy as np
    import ded_inputs as di
    import oracle
    from paper_2407_12021_amd import binding as B
    tri = di.SyntheticTrigram(32000, seed=0)
    g = np.random.default_rng(5)
    prev, root = 17, 4711
    cands = []
    for _ in range(24):
        a, b, seq = prev, root, []
        for _ in range(4):
            succ, prob = tri.successors(a, b)
            t = int(succ[g.choice(len(succ), p=prob)])
            seq.append(t)
            a, b = b, t
        cands.append(seq)
    rc, parent, token, end = B.ded_build_tree(root, cands, 1 + 24 * 4)
    assert rc == B.DED_OK and len(parent) <= 97
    assert (parent.tolist(), token.tolist(), end.tolist()) == oracle.build_trie(root, cands, 97)
    cfg = B.make_config(2, 256, 4, 4, 64, 512, 32000, 10000.0, 1e-5, "fp32", 1, 256, 128)
    assert B.ded_validate_tree(cfg, [10], [len(parent)], np.pad(parent, (0, 128 - len(parent)))[None],
                               np.pad(token, (0, 128 - len(token)))[None]) == B.DED_OK
    # argument errors
    lib = B.lib()
    import ctypes as C
    one = (C.c_int32 * 4)()
    assert lib.ded_build_tree(1, 1, one, one, 4, 0, one, one, one, one) == B.DED_EINVAL        # no room for the root
    assert lib.ded_build_tree(1, -1, one, one, 4, 4, one, one, one, one) == B.DED_EINVAL
    assert lib.ded_build_tree(1, 1, one, one, 4, 4, None, one, one, one) == B.DED_EINVAL
    bad = (C.c_int32 * 1)(5)
    assert lib.ded_build_tree(1, 1, bad, one, 4, 4, one, one, one, one) == B.DED_EINVAL        # length above max_len


def test_sample_rejects_null_context():
    import ctypes as C
    from paper_2407_12021_amd import binding as B
    u = (C.c_float * 4)()
    assert B.lib().ded_sample(None, 1.0, 0.9, u) == B.DED_EINVAL


def test_library_is_loaded_after_torch(b):
    """torch brings its own HIP runtime; the library has to find that one already in the process (loaded the
    other way round, device pointers allocated by torch are foreign to the runtime the library pulls in).
    A host-only call must therefore not be able to load the library before torch."""
    import subprocess
    import sys
    code = ("import sys; from paper_2407_12021_amd import binding as B; assert 'torch' not in sys.modules; "
            "rc, parent, token, end = B.ded_build_tree(7, [[1, 2]], 8); assert rc == 0 and len(parent) == 3; "
            "assert 'torch' in sys.modules")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]


def test_host_api_from_plain_c(b, tmp_path):
    """tests/c/host_api.c, compiled with gcc against include/ded_verify.h and linked to the shared library, drives
    the host-only entry points (draft maker, pseudo-sequence, validation) without Python in between."""
    import subprocess
    exe = str(tmp_path / "host_api")
    lib_dir = os.path.dirname(b.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c", "host_api.c"), "-o", exe, "-L", lib_dir, "-lded_verify",
           "-Wl,-rpath," + lib_dir, "-Wl,-rpath,/opt/rocm/lib", "-L", "/opt/rocm/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), (r.stdout[-2000:], r.stderr[-2000:])
