"""GPU end-to-end parity of the C-ABI decode path against the CPU oracle."""
import dataclasses

import numpy as np
import pytest

import workload as wl
import oracle
from oracle.llama import as_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2408_15766_amd as P
    assert torch.cuda.is_available()
    return torch, P


@pytest.fixture(scope="module")
def tiny_gpu(env):
    torch, P = env
    sh = wl.TINY
    hw = wl.make_weights(sh)
    return sh, hw, as_dtype(hw, np.float64), wl.make_prompt(sh), P.upload_weights(hw, sh.dtype)


def oracle_tree_to_gpu(P, t, cap):
    g = P.Tree.empty(cap)
    n = t.n_nodes
    g.token[:n], g.parent[:n], g.depth[:n], g.score[:n] = t.token, t.parent, t.depth, t.score
    g.n_nodes = n
    return g


def test_tiny_fp32_greedy_matches_oracle_token_for_token(env, tiny_gpu):
    """Plain decoding through the same kernels (tree of the root alone)."""
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    eng = P.Engine(sh, dw, tree=(1, 1, 1))
    got, taus = eng.generate(prompt, sh.gen_tokens)
    want = oracle.greedy_decode(w64, sh, prompt, sh.gen_tokens)
    assert got == want and set(taus) == {1}


def test_tiny_fp32_spec_matches_oracle_per_cycle(env, tiny_gpu):
    """Config 0: tokens identical, the draft tree identical, logits within 1e-4, features, KV cache."""
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    eng = P.Engine(sh, dw)
    grec, orec = [], []
    got, gt = eng.generate(prompt, sh.gen_tokens, record=grec)
    want, wt = oracle.spec_decode(w64, sh, prompt, sh.gen_tokens, record=orec)
    assert got == want == oracle.greedy_decode(w64, sh, prompt, sh.gen_tokens)
    assert gt == wt
    assert len(grec) == len(orec)
    for a, b in zip(grec, orec):
        ta, tb = a["tree"], b["tree"]
        assert ta.n_nodes == tb.n_nodes == sh.tree_total
        assert list(ta.token) == list(tb.token) and list(ta.parent) == list(tb.parent) and list(ta.depth) == list(tb.depth)
        assert np.abs(ta.score - tb.score).max() < 2e-5
        assert np.abs(a["logits"] - b["logits"]).max() < 1e-4
        assert np.abs(a["feats"] - b["feats"]).max() < 1e-4


@pytest.mark.parametrize("shape", [(1, 1, 2), (2, 3, 5), (15, 1, 16), (3, 16, 40), (6, 10, 60), (15, 16, 128)],
                         ids=lambda s: "D%d-K%d-N%d" % s)
def test_tiny_fp32_tree_shapes_match_oracle(env, tiny_gpu, shape):
    """Other tree shapes, up to the largest the library accepts (depth 15, top-k 16, 128 verified rows: a pool of
    3600 candidates) and down to a single draft token: tokens, trees and logits against the oracle per cycle."""
    torch, P = env
    sh0, hw, w64, prompt, dw = tiny_gpu
    D, K, N = shape
    gen = 20
    sh = sh0.with_(tree_depth=D, tree_topk=K, tree_total=N, gen_tokens=gen)
    eng = P.Engine(sh, dw)
    grec, orec = [], []
    got, gt = eng.generate(prompt, gen, record=grec)
    want, wt = oracle.spec_decode(w64, sh, prompt, gen, record=orec)
    assert got == want and gt == wt and len(grec) == len(orec)
    for a, b in zip(grec, orec):
        ta, tb = a["tree"], b["tree"]
        assert ta.n_nodes == tb.n_nodes == N
        assert list(ta.token) == list(tb.token) and list(ta.parent) == list(tb.parent) and list(ta.depth) == list(tb.depth)
        assert np.abs(ta.score - tb.score).max() < 5e-5
        assert np.abs(a["logits"] - b["logits"]).max() < 1e-4


def assert_committed_rows_equal_plain(srec, prec):
    """Every row of a speculative cycle that gets committed (the root and each accepted node) carries, bit for bit, the
    logits plain decoding produced for the same position: the accepted node of depth d of a cycle that started with n
    committed tokens sits at position n + d, where plain decoding ran its single row when it had n + d tokens committed."""
    plain_at = {r["n"]: r["logits"][0] for r in prec}
    checked = deeper = 0
    for r in srec:
        t, cur = r["tree"], 0
        nodes = [0]
        for tok in r["emitted"][:-1]:                          # the accepted tokens; the last emitted one is the bonus
            cur = next(c for c in range(cur + 1, t.n_nodes) if t.parent[c] == cur and t.token[c] == tok)
            nodes.append(cur)
        for d, node in enumerate(nodes):
            if r["n"] + d in plain_at:
                assert np.array_equal(r["logits"][node], plain_at[r["n"] + d]), (r["n"], d, node)
                checked += 1
                deeper += d > 0
    return checked, deeper


def forge_hook(stream, n_prompt, plan, rng, vocab):
    """Graft the known continuation into the GPU-drafted tree (host arrays of the C ABI)."""
    def hook(eng, t):
        n = eng.committed
        k = n - n_prompt + 1
        want = plan(n)
        nn = t.n_nodes
        tok, par = t.token, t.parent
        cur, on_path = 0, {0}
        for d in range(1, want + 1):
            if k + d - 1 >= len(stream):
                break
            kids = [c for c in range(nn) if par[c] == cur]
            if kids:
                c = kids[int(rng.integers(len(kids)))]
            else:
                leaves = [c for c in range(cur + 1, nn) if c not in on_path and not any(par[x] == c for x in range(nn))]
                if not leaves:
                    break
                c = leaves[int(rng.integers(len(leaves)))]
                par[c] = cur
            tok[c] = stream[k + d - 1]
            cur = c
            on_path.add(c)
        for j in range(1, nn):
            t.depth[j] = t.depth[par[j]] + 1
        return t
    return hook


@pytest.mark.parametrize("want", [1, 2, 3])
def test_tiny_fp32_forged_trees_accept_and_compact(env, tiny_gpu, want):
    """Forged trees force acceptance lengths 1..D; output must stay the greedy stream, and the compacted
    KV cache must equal the oracle's cache for the committed sequence."""
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    gen = 40
    greedy = oracle.greedy_decode(w64, sh, prompt, gen + 8)
    eng = P.Engine(sh, dw)
    rng = np.random.default_rng(want)
    got, taus = eng.generate(prompt, gen, tree_hook=forge_hook(greedy, len(prompt), lambda n: want, rng, sh.vocab))
    assert got == greedy[:gen]
    assert max(taus) == want + 1 and min(taus) >= 1
    n = eng.committed
    seq = np.array(list(prompt) + greedy)[:n]
    ref = oracle.KVCache(sh.n_layers, n, sh.n_kv_heads, sh.head_dim)
    _, feats = oracle.target_forward(w64, sh, ref, seq, np.arange(n), list(range(n)), [list(range(i + 1)) for i in range(n)])
    for l in range(sh.n_layers):
        k, v = eng.kv(0, l, n)
        assert np.abs(k - ref.k[l].reshape(n, -1)).max() < 1e-4
        assert np.abs(v - ref.v[l].reshape(n, -1)).max() < 1e-4
    # draft cache: one entry per committed token except the first, all from true target features
    dref = oracle.KVCache(1, n + 1, sh.n_kv_heads, sh.head_dim)
    pos = np.arange(1, n)
    oracle.draft_forward(w64, sh, dref, feats[:-1], seq[1:], pos, list(pos), [list(range(1, p + 1)) for p in pos])
    n_d = n - (taus[-1])                      # entries written by root steps so far: up to the last cycle's old n
    k, v = eng.kv(1, 0, n_d)
    assert np.abs(k - dref.k[0, 1:n_d + 1].reshape(n_d, -1)).max() < 1e-4
    assert np.abs(v - dref.v[0, 1:n_d + 1].reshape(n_d, -1)).max() < 1e-4


def test_tiny_fp32_sampling_matches_oracle_decisions(env, tiny_gpu):
    """T = 1 with the shared counter-based RNG: same seed -> same tokens as the oracle."""
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    for seed in (1, 2):
        eng = P.Engine(sh, dw, temperature=1.0, seed=seed)
        got, gt = eng.generate(prompt, 24)
        want, wt = oracle.spec_decode(w64, sh, prompt, 24, temperature=1.0, seed=seed)
        assert got == want and gt == wt


def test_tiny_fp32_sampling_accept_matches_oracle_on_forged_peaky_tree(env, tiny_gpu):
    """Rejection sampling where acceptance actually happens: verify an oracle-forged tree whose children carry
    the target's most probable tokens, at a low temperature, for several seeds."""
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    temp = 0.05
    accepted_any = False
    for seed in range(6):
        st, first = oracle.prefill(w64, sh, prompt, 128, temp, seed)
        st.cycle = 1
        t = oracle.draft_tree(st, sh.tree_depth, sh.tree_topk, sh.tree_total)
        # first pass to learn the target's favourites, then plant them as children of the root and of node 1
        lg, _ = oracle.verify_tree(st, t)
        fav0 = oracle.top_k(lg[0], 3)
        kids0 = t.children(0)[:3]
        for c, v in zip(kids0, fav0):
            t.token[c] = v
        lg, ft = oracle.verify_tree(st, t)
        acc, bonus = oracle.accept_sample(t, lg, temp, seed, 1)
        eng = P.Engine(sh, dw, temperature=temp, seed=seed)
        assert eng.prefill(prompt) == first
        eng.draft_tree()
        g = oracle_tree_to_gpu(P, t, sh.tree_total)
        eng.verify(g)
        out = eng.accept(g)
        assert out == [int(t.token[j]) for j in acc] + [bonus]
        accepted_any |= len(acc) > 0
    assert accepted_any


def test_call_order_malformed_trees_and_capacity_are_reported(env, tiny_gpu):
    """Error paths of the C ABI: calls out of order, trees that are not trees, a full cache.  Every failure is an
    error code with a message; nothing is launched for a rejected call and the context keeps working."""
    torch, P = env
    B = P.binding
    sh, hw, w64, prompt, dw = tiny_gpu
    eng = P.Engine(sh, dw)

    def code(fn, *a):
        with pytest.raises(B.SpecError) as e:
            fn(*a)
        assert str(e.value)
        return e.value.code

    t0 = P.Tree.empty(sh.tree_total)
    assert code(eng.draft_tree) == B.SPEC_ESTATE                  # before prefill
    assert code(eng.verify, t0) == B.SPEC_ESTATE
    assert code(eng.accept, t0) == B.SPEC_ESTATE
    assert code(eng.prefill, []) == B.SPEC_EINVAL
    assert code(eng.prefill, [sh.vocab]) == B.SPEC_EINVAL         # token out of range
    first = eng.prefill(prompt)
    assert code(eng.accept, t0) == B.SPEC_ESTATE                  # nothing verified yet
    t = eng.draft_tree()
    good = (t.token.copy(), t.parent.copy(), t.depth.copy(), t.n_nodes)

    def restore():
        t.token[:], t.parent[:], t.depth[:], t.n_nodes = good[0], good[1], good[2], good[3]

    for edit in ("root", "parent_after", "depth", "token", "count0", "count_big", "too_deep"):
        restore()
        if edit == "root": t.token[0] = (first + 1) % sh.vocab
        if edit == "parent_after": t.parent[2] = 5
        if edit == "depth": t.depth[3] += 1
        if edit == "token": t.token[4] = -1
        if edit == "count0": t.n_nodes = 0
        if edit == "count_big": t.n_nodes = sh.tree_total + 1
        if edit == "too_deep":
            for j in range(1, 16): t.parent[j] = j - 1            # a 15-deep chain is fine ...
            for j in range(1, 16): t.depth[j] = j
            t.depth[15] = 16                                      # ... a claimed depth of 16 is not
        assert code(eng.verify, t) == B.SPEC_EINVAL, edit
    restore()
    eng.verify(t)                                                 # the context is still in the DRAFTED state
    assert code(eng.verify, t) == B.SPEC_ESTATE
    want = oracle.greedy_decode(w64, sh, prompt, 8)
    out = [first] + eng.accept(t)
    assert out == want[:len(out)]
    eng.close()

    # capacity: room for the prompt, one tree and two more tokens
    eng = P.Engine(sh, dw, max_seq=len(prompt) + sh.tree_total + 2)
    toks = [eng.prefill(prompt)]
    seen = None
    for _ in range(6):
        try:                                                      # the draft call already refuses a cycle that cannot fit
            t = eng.draft_tree()
            eng.verify(t)
        except B.SpecError as e:
            seen = e.code
            break
        toks += eng.accept(t)
    assert seen == B.SPEC_ECAP and toks == want[:len(toks)]
    eng.close()


def test_tiny_fp32_partial_tree_matches_oracle(env, tiny_gpu):
    """A caller may verify fewer nodes than the configured total (a prefix of the drafted tree is a tree): logits,
    acceptance and the following cycles agree with the oracle run on the same truncated trees."""
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    eng = P.Engine(sh, dw)
    keep = [7, 1, 16, 3, 11]
    hook_calls = []

    def gpu_hook(e, t):
        t.n_nodes = keep[len(hook_calls) % len(keep)]
        hook_calls.append(t.n_nodes)
        return t

    ocalls = []

    def oracle_hook(st, t):
        k = keep[len(ocalls) % len(keep)]
        ocalls.append(k)
        return oracle.Tree(t.token[:k].copy(), t.parent[:k].copy(), t.depth[:k].copy(), t.score[:k].copy())

    grec, orec = [], []
    got, gt = eng.generate(prompt, 24, tree_hook=gpu_hook, record=grec)
    want, wt = oracle.spec_decode(w64, sh, prompt, 24, tree_hook=oracle_hook, record=orec)
    assert got == want and gt == wt and hook_calls == ocalls
    for a, b in zip(grec, orec):
        assert a["tree"].n_nodes == b["tree"].n_nodes
        assert np.abs(a["logits"] - b["logits"]).max() < 1e-4


BF16_TRUNC = wl.LLAMA2_7B.with_(name="llama2-7b-2layer", n_layers=2, prompt_len=96, gen_tokens=24)
BF16_GQA = wl.LLAMA3_8B.with_(name="llama3-8b-width-2layer", n_layers=2, vocab=8192, d_ffn=4096, prompt_len=300, gen_tokens=16)


@pytest.fixture(scope="module", params=[BF16_TRUNC, BF16_GQA], ids=lambda s: s.name)
def bf16_model(request, env):
    torch, P = env
    sh = request.param
    hw = wl.make_weights(sh)
    return sh, hw, P.upload_weights(hw, sh.dtype), wl.make_prompt(sh)


# Ceilings of the bf16 logit comparisons, set above what the kernels measure on these models.  Against the bf16-storage
# evaluation of the oracle: rms 0.0059 .. 0.0063; the maximum over 0.5 .. 1.9 million logits is the tail of that noise
# and moves between 0.029 and 0.035 with any change of rounding order (the binding requirement is the per-logit
# tolerance itself, which every logit meets).  Against the plain oracle: maximum 0.067 .. 0.074, rms 0.0129 .. 0.0137,
# 99.56 .. 99.70 % inside the tolerance.
STORE_MAX, STORE_RMS = 0.038, 0.0068
PLAIN_MAX, PLAIN_RMS, PLAIN_INSIDE = 0.080, 0.0145, 0.995


def oracle_logits_for(hw, sh, prompt, t, first, dtype, store):
    st, _ = oracle.prefill(as_dtype(hw, dtype), sh, prompt, len(prompt) + 200, dtype=dtype, store=store)
    ot = oracle.Tree(t.token[:t.n_nodes].copy(), t.parent[:t.n_nodes].copy(), t.depth[:t.n_nodes].copy(), t.score[:t.n_nodes].copy())
    ot.token[0] = first                       # compare on the GPU's root token even if a near-tie flipped the oracle's
    return np.asarray(oracle.verify_tree(st, ot)[0], dtype=np.float64)


def logit_stats(name, x, ref, tag):
    err = np.abs(x - ref)
    ok = err <= 3e-2 + 2e-2 * np.abs(ref)
    print(f"{name} {tag}: max err {err.max():.4f} rms {np.sqrt((err ** 2).mean()):.4f} within tolerance {ok.mean() * 100:.4f} %")
    return err.max(), np.sqrt((err ** 2).mean()), ok


def test_bf16_logits_within_tolerance_of_oracle(env, bf16_model):
    """Real widths, two layers: GPU bf16 logits of a verified tree against the oracle on the same tree.

    Tolerance per logit: 3e-2 + 2e-2 |ref|, required of EVERY logit.

    The reference is the oracle evaluated with the configuration's storage type: `store=round_to_bf16` rounds the
    tensors that a bf16 configuration holds in memory between two operations (norm outputs, cached keys and values,
    the attention output, the SwiGLU output, the features) and leaves the residual stream, the queries and every
    accumulation in fp64.  Those are the storage points of this library's kernels, so this reading describes what
    the kernels are meant to compute; the oracle's default (no rounding anywhere) stays the plain definition.
    Against that plain definition the tolerance cannot hold for every logit once keys, values and GEMM inputs are
    bf16 (rounding the cached keys and values alone moves single logits by more than 0.03 at a logit spread of 1.3);
    that comparison is reported and held to fixed ceilings as a regression guard."""
    torch, P = env
    sh, hw, dw, prompt = bf16_model
    eng = P.Engine(sh, dw)
    first = eng.prefill(prompt)
    t = eng.draft_tree()
    eng.verify(t)
    got = eng.logits(t.n_nodes)
    g_max, g_rms, ok = logit_stats(sh.name, got, oracle_logits_for(hw, sh, prompt, t, first, np.float64, wl.round_to_bf16),
                                   "GPU vs oracle with bf16 storage")
    assert ok.all()
    assert g_max <= STORE_MAX and g_rms <= STORE_RMS
    p_max, p_rms, p_ok = logit_stats(sh.name, got, oracle_logits_for(hw, sh, prompt, t, first, np.float32, None),
                                     "GPU vs plain fp32 oracle (informational)")
    assert p_ok.mean() >= PLAIN_INSIDE and p_max < PLAIN_MAX and p_rms < PLAIN_RMS


def test_bf16_prefill_in_several_tiles_matches_oracle(env):
    """A 300-token prompt at 7B width runs the prefill projections as three 128-row tiles (the last one ragged), with
    SwiGLU formed inside the tiled gate/up launch; the logits of the following verify depend on every cached key and
    value, and are compared with the bf16-storage oracle like in the test above."""
    torch, P = env
    sh = wl.LLAMA2_7B.with_(name="llama2-7b-2layer-p300", n_layers=2, prompt_len=300, gen_tokens=8)
    hw = wl.make_weights(sh)
    dw = P.upload_weights(hw, sh.dtype)
    prompt = wl.make_prompt(sh)
    eng = P.Engine(sh, dw)
    first = eng.prefill(prompt)
    t = eng.draft_tree()
    eng.verify(t)
    g_max, g_rms, ok = logit_stats(sh.name, eng.logits(t.n_nodes), oracle_logits_for(hw, sh, prompt, t, first, np.float64, wl.round_to_bf16),
                                   "GPU vs oracle with bf16 storage")
    assert ok.all() and g_max <= STORE_MAX and g_rms <= STORE_RMS


LONG_PROMPT = [wl.LLAMA2_7B.with_(name="llama2-7b-2layer-p1400", n_layers=2, prompt_len=1400, gen_tokens=8),
               wl.LLAMA3_8B.with_(name="llama3-8b-width-2layer-p1400", n_layers=2, vocab=8192, d_ffn=4096, prompt_len=1400, gen_tokens=8)]


@pytest.mark.parametrize("sh", LONG_PROMPT, ids=lambda s: s.name)
def test_bf16_logits_long_prompt_within_tolerance_of_oracle(env, sh):
    """A 1400-token prompt: every verified row's attention runs eight 128-key parts and the 256-key parts beyond
    position 1024 on the matrix cores (and the prefill three 512-row chunks), MHA 32 x 128 and GQA 32 / 8; the logits
    of the verified tree against the bf16-storage oracle, every logit inside the tolerance."""
    torch, P = env
    hw = wl.make_weights(sh)
    dw = P.upload_weights(hw, sh.dtype)
    prompt = wl.make_prompt(sh)
    eng = P.Engine(sh, dw)
    first = eng.prefill(prompt)
    t = eng.draft_tree()
    eng.verify(t)
    g_max, g_rms, ok = logit_stats(sh.name, eng.logits(t.n_nodes), oracle_logits_for(hw, sh, prompt, t, first, np.float64, wl.round_to_bf16),
                                   "GPU vs oracle with bf16 storage")
    assert ok.all() and g_max <= STORE_MAX and g_rms <= STORE_RMS


def test_bf16_spec_equals_greedy_bit_exact(env, bf16_model):
    """GPU speculative decoding == GPU plain decoding, token for token and logit bit for logit bit,
    with the real (random) draft and with forged trees that force acceptance."""
    torch, P = env
    sh, hw, dw, prompt = bf16_model
    gen = sh.gen_tokens
    plain = P.Engine(sh, dw, tree=(1, 1, 1))
    prec = []
    greedy, _ = plain.generate(prompt, gen + 8, record=prec)
    spec = P.Engine(sh, dw)
    got, taus = spec.generate(prompt, gen)
    assert got == greedy[:gen]
    rng = np.random.default_rng(0)
    spec2 = P.Engine(sh, dw)
    srec = []
    got2, taus2 = spec2.generate(prompt, gen, tree_hook=forge_hook(greedy, len(prompt), lambda n: n % 5, rng, sh.vocab), record=srec)
    assert got2 == greedy[:gen] and max(taus2) >= 4
    # logits of every committed row (root and accepted nodes) == logits plain decoding produced at that position
    checked, deeper = assert_committed_rows_equal_plain(srec, prec)
    assert checked >= len(srec) and deeper >= 3


@pytest.mark.parametrize("shape", [(15, 16, 128), (8, 10, 80), (2, 4, 7)], ids=lambda s: "D%d-K%d-N%d" % s)
def test_bf16_other_tree_shapes_equal_greedy_bit_exact(env, bf16_model, shape):
    """The bit-exactness argument does not depend on the tree shape: trees of 80 and 128 rows (three and four
    32-row token tiles in the GEMM, more query blocks in the attention) and a tiny one, forged to accept up to
    the tree's depth, emit the plain-decoding stream and the same root-row logits."""
    torch, P = env
    sh0, hw, dw, prompt = bf16_model
    D, K, N = shape
    sh = sh0.with_(tree_depth=D, tree_topk=K, tree_total=N)
    gen = 20
    cap = len(prompt) + gen + D + N + 40
    plain = P.Engine(sh, dw, tree=(1, 1, 1), max_seq=cap)
    prec = []
    greedy, _ = plain.generate(prompt, gen + D + 2, record=prec)
    rng = np.random.default_rng(1)
    spec = P.Engine(sh, dw, max_seq=cap)
    srec = []
    got, taus = spec.generate(prompt, gen, tree_hook=forge_hook(greedy, len(prompt), lambda n: n % (min(D, 6) + 1), rng, sh.vocab), record=srec)
    assert got == greedy[:gen] and max(taus) >= min(D, 3)
    checked, deeper = assert_committed_rows_equal_plain(srec, prec)
    assert checked >= len(srec) and deeper >= min(D, 3) - 1


def test_graph_replay_equals_eager_launches(env, bf16_model):
    """The verify forward replayed from a HIP graph gives the same bits as individually launched kernels,
    on every cycle, with eager work (draft, accept, host syncs) between the replays."""
    torch, P = env
    sh, hw, dw, prompt = bf16_model
    gen = 12
    plain = P.Engine(sh, dw, tree=(1, 1, 1), graphs=False)
    greedy, _ = plain.generate(prompt, gen + 8)
    outs = []
    for graphs in (True, False):
        rng = np.random.default_rng(4)
        eng = P.Engine(sh, dw, graphs=graphs)
        rec = []
        toks, taus = eng.generate(prompt, gen, tree_hook=forge_hook(greedy, len(prompt), lambda n: n % 3, rng, sh.vocab), record=rec)
        outs.append((toks, taus, rec))
    (ta, ua, ra), (tb, ub, rb) = outs
    assert ta == tb == greedy[:gen] and ua == ub and len(ra) == len(rb) >= 4
    for a, b in zip(ra, rb):
        assert np.array_equal(a["logits"], b["logits"]) and np.array_equal(a["feats"], b["feats"])


def test_results_do_not_depend_on_workspace_contents(env, bf16_model, tiny_gpu):
    """The library initialises everything it reads: a workspace handed over full of 0xFF bytes (NaN patterns in
    bf16 and fp32) gives bit-identical trees, tokens and logits to a zero-filled one.  Also with a one-token
    prompt, where the draft cache is empty in the first cycle."""
    torch, P = env
    cases = [(bf16_model[0], bf16_model[2], bf16_model[3]), (tiny_gpu[0], tiny_gpu[4], tiny_gpu[3]),
             (tiny_gpu[0], tiny_gpu[4], tiny_gpu[3][:1])]
    for sh, dw, prompt in cases:
        runs = []
        for fill in (0, 0xFF):
            eng = P.Engine(sh, dw, workspace_fill=fill)
            rec = [eng.prefill(prompt)]
            for _ in range(4):
                t = eng.draft_tree()
                eng.verify(t)
                rec.append((t.token[:t.n_nodes].copy(), t.parent[:t.n_nodes].copy(), t.score[:t.n_nodes].copy(),
                            eng.logits(t.n_nodes).copy(), list(eng.accept(t))))
            eng.close()
            runs.append(rec)
        assert runs[0][0] == runs[1][0]
        for a, b in zip(runs[0][1:], runs[1][1:]):
            assert all(np.array_equal(x, y) for x, y in zip(a[:4], b[:4])) and a[4] == b[4]
            assert np.isfinite(a[3]).all()


def test_bf16_sampling_acceptance_matches_oracle_on_gpu_logits(env, bf16_model):
    """T = 1 at real vocabulary sizes (the LLaMA2-13B configuration's mode): the GPU's rejection-sampling
    decisions must equal the oracle's acceptance run on the GPU's own fp32 logits, cycle by cycle."""
    torch, P = env
    sh, hw, dw, prompt = bf16_model
    temp = 1.0
    for seed in (11, 12):
        eng = P.Engine(sh, dw, temperature=temp, seed=seed)
        eng.prefill(prompt)
        for cycle in range(1, 5):
            t = eng.draft_tree()
            eng.verify(t)
            lg = eng.logits(t.n_nodes)
            ot = oracle.Tree(t.token[:t.n_nodes].copy(), t.parent[:t.n_nodes].copy(), t.depth[:t.n_nodes].copy(), t.score[:t.n_nodes].copy())
            acc, bonus = oracle.accept_sample(ot, lg, temp, seed, cycle)
            assert eng.accept(t) == [int(ot.token[j]) for j in acc] + [bonus]
    # low temperature: the distribution is peaky, rejection tests are decided by real probabilities
    eng = P.Engine(sh, dw, temperature=0.3, seed=5)
    eng.prefill(prompt)
    for cycle in range(1, 4):
        t = eng.draft_tree()
        eng.verify(t)
        lg = eng.logits(t.n_nodes)
        ot = oracle.Tree(t.token[:t.n_nodes].copy(), t.parent[:t.n_nodes].copy(), t.depth[:t.n_nodes].copy(), t.score[:t.n_nodes].copy())
        acc, bonus = oracle.accept_sample(ot, lg, 0.3, 5, cycle)
        assert eng.accept(t) == [int(ot.token[j]) for j in acc] + [bonus]


LONG_GQA = wl.LLAMA3_8B.with_(name="llama3-8b-width-2layer-long", n_layers=2, vocab=8192, d_ffn=4096, prompt_len=4096, gen_tokens=12)


def test_long_context_spec_equals_greedy_bit_exact(env):
    """The LLaMA3-8B configuration's long-KV verify (4096-token prompt, GQA 32/8): speculative decoding with
    forged acceptance equals plain decoding token for token and in the root row's logit bits."""
    torch, P = env
    sh = LONG_GQA
    dw = P.pack_weights(wl.iter_device_weights(sh, "cuda"))
    prompt = wl.make_prompt(sh)
    gen = sh.gen_tokens
    plain = P.Engine(sh, dw, tree=(1, 1, 1))
    prec = []
    greedy, _ = plain.generate(prompt, gen + 8, record=prec)
    rng = np.random.default_rng(1)
    spec = P.Engine(sh, dw)
    srec = []
    got, taus = spec.generate(prompt, gen, tree_hook=forge_hook(greedy, len(prompt), lambda n: (n * 7) % 6, rng, sh.vocab), record=srec)
    assert got == greedy[:gen] and max(taus) >= 4
    checked, deeper = assert_committed_rows_equal_plain(srec, prec)
    assert checked >= len(srec) and deeper >= 3


def test_full_depth_7b_bench_configuration(env):
    """BASELINE's LLaMA2-7B configuration at full size, in the launch configuration bench.py times (device-drawn
    weights, graph replay): (1) speculative == plain decoding for 12 tokens with forged acceptance; (2) sampled
    logits of the LM head equal the oracle's dot products of the GPU's feature rows with the head's rows."""
    torch, P = env
    sh = wl.LLAMA2_7B
    named = dict(wl.iter_device_weights(sh, "cuda"))
    head_rows = {v: named["lm_head"][v].float().cpu().numpy() for v in (0, 1, 777, 31999)}
    dw = P.pack_weights(named.items())
    del named
    prompt = wl.make_prompt(sh)
    gen = 12
    plain = P.Engine(sh, dw, tree=(1, 1, 1))
    greedy, _ = plain.generate(prompt, gen + 8)
    rng = np.random.default_rng(2)
    spec = P.Engine(sh, dw)
    rec = []
    got, taus = spec.generate(prompt, gen, tree_hook=forge_hook(greedy, len(prompt), lambda n: n % 4, rng, sh.vocab), record=rec)
    assert got == greedy[:gen] and max(taus) >= 3
    r = rec[-1]
    for v, w_row in head_rows.items():
        want = r["feats"].astype(np.float64) @ w_row.astype(np.float64)
        assert np.abs(r["logits"][:, v] - want).max() < 2e-3
