"""Host-side checks that need no GPU: the library loads, exports every declared symbol, and its
host-only entry points validate their arguments."""
import ctypes as C
import os
import re

import numpy as np

import pytest

import workload as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    import paper_2408_15766_amd as pkg
    return pkg


def declared_symbols():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not h.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(spec_[a-z_0-9]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol(P):
    names = declared_symbols()
    assert {"spec_create", "spec_prefill", "spec_draft_tree", "spec_verify", "spec_accept", "spec_destroy",
            "spec_k_gemm", "spec_hca_attention"} <= names
    for n in sorted(names):
        assert hasattr(P.lib, n), f"libspec.so does not export {n}"


def make_cfg(P, sh, **kw):
    b = P.binding
    vals = dict(n_layers=sh.n_layers, d_model=sh.d_model, n_q_heads=sh.n_q_heads, n_kv_heads=sh.n_kv_heads, head_dim=sh.head_dim,
                d_ffn=sh.d_ffn, vocab=sh.vocab, rope_theta=sh.rope_theta, rms_eps=sh.rms_eps, dtype=1 if sh.dtype == "bf16" else 0,
                max_seq=sh.prompt_len + sh.gen_tokens + sh.tree_total + 8, tree_depth=sh.tree_depth, tree_topk=sh.tree_topk,
                tree_total=sh.tree_total, temperature=0.0, seed=0, device=0, stream=None, workspace=None, workspace_bytes=0)
    vals.update(kw)
    return b.spec_config(**vals)


def test_workspace_bytes_all_configs(P):
    sizes = {}
    for sh in wl.CONFIGS:
        n = P.spec_workspace_bytes(make_cfg(P, sh))
        assert n > 0 and n % 256 == 0
        sizes[sh.name] = n
        esz = 2 if sh.dtype == "bf16" else 4
        kv = sh.n_layers * 2 * (sh.prompt_len + sh.gen_tokens + sh.tree_total + 8) * sh.d_kv * esz
        assert n > kv                                   # holds at least the target KV cache
    assert sizes["llama3-70b"] < 2e9                    # caches + scratch stay far below the 288 GB of HBM


@pytest.mark.parametrize("kw", [dict(dtype=7), dict(head_dim=80), dict(n_q_heads=6, n_kv_heads=4), dict(tree_total=0),
                                dict(tree_total=129), dict(tree_depth=16), dict(tree_topk=17), dict(max_seq=4),
                                dict(temperature=-1.0), dict(d_model=255), dict(vocab=0)])
def test_invalid_config_is_rejected(P, kw):
    cfg = make_cfg(P, wl.TINY, **kw)
    assert P.spec_workspace_bytes(cfg) == 0
    out = C.c_void_p()
    w = P.binding.spec_weights()
    assert P.lib.spec_create(C.byref(cfg), C.byref(w), C.byref(out)) == P.binding.SPEC_EINVAL
    assert not out.value and "configuration" in P.spec_last_error(None)


def test_create_rejects_null_weights_and_small_workspace(P):
    cfg = make_cfg(P, wl.TINY)
    out = C.c_void_p()
    w = P.binding.spec_weights()
    assert P.lib.spec_create(C.byref(cfg), C.byref(w), C.byref(out)) == P.binding.SPEC_EINVAL
    assert P.lib.spec_create(C.byref(cfg), None, C.byref(out)) == P.binding.SPEC_EINVAL
    assert P.lib.spec_create(None, C.byref(w), C.byref(out)) == P.binding.SPEC_EINVAL
    assert P.lib.spec_create(C.byref(cfg), C.byref(w), None) == P.binding.SPEC_EINVAL


def test_null_context_calls_do_not_crash(P):
    assert P.lib.spec_prefill(None, None, 0, None) == P.binding.SPEC_EINVAL
    assert P.lib.spec_draft_tree(None, None) == P.binding.SPEC_EINVAL
    assert P.lib.spec_verify(None, None) == P.binding.SPEC_EINVAL
    assert P.lib.spec_accept(None, None, None, None) == P.binding.SPEC_EINVAL
    assert P.lib.spec_committed(None) == P.binding.SPEC_EINVAL
    P.lib.spec_destroy(None)
    assert P.lib.spec_k_gemm(0, None, 0, 0, 0, None, 0, None, 0, None, 0, None, 0, 0, 0, None) == P.binding.SPEC_EINVAL


def test_algorithmic_bytes_match_shape_arithmetic():
    b = wl.algorithmic_bytes(wl.LLAMA2_7B)
    assert abs(b["verify_weights"] / 1e9 - 13.21) < 0.01 and b["kv_bytes_per_token"] == 524288
    b = wl.algorithmic_bytes(wl.LLAMA3_70B)
    assert abs(b["verify_weights"] / 1e9 - 139.0) < 0.1 and b["kv_bytes_per_token"] == 327680


def test_graft_continuation_keeps_the_tree_valid():
    """Host-side input preparation used by the benchmark's teacher-forced mode: after grafting, parents still precede
    children, depths are consistent, and the continuation is a root-to-node path."""
    import workload as wl
    rng = np.random.default_rng(0)
    for trial in range(50):
        n = int(rng.integers(2, 61))
        parent = np.full(64, -1, dtype=np.int32)
        for j in range(1, n):
            parent[j] = int(rng.integers(0, min(j, 1 + j // 3) if trial % 2 else j))
        depth = np.zeros(64, dtype=np.int32)
        for j in range(1, n):
            depth[j] = depth[parent[j]] + 1
        token = rng.integers(0, 1000, size=64).astype(np.int32)
        cont = [int(x) for x in rng.integers(1000, 2000, size=int(rng.integers(0, 7)))]
        done = wl.graft_continuation(token, parent, depth, n, cont)
        assert 0 <= done <= len(cont) and parent[0] == -1 and depth[0] == 0
        cur = 0
        for d in range(done):
            kids = [c for c in range(n) if parent[c] == cur and token[c] == cont[d]]
            assert kids
            cur = kids[0]
        for j in range(1, n):
            assert 0 <= parent[j] < j and depth[j] == depth[parent[j]] + 1
