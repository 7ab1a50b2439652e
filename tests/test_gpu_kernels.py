"""GPU parity of the individual kernels (through the C ABI) against the CPU oracle's functions."""
import zlib

import numpy as np
import pytest

import workload as wl
from oracle import attention_row, log_softmax, top_k

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2408_15766_amd as P
    assert torch.cuda.is_available()
    return torch, P


def case_seed(*case):
    """A fixed seed per test case (the built-in hash of a tuple with a string in it changes from process to process)."""
    return zlib.crc32(repr(case).encode())


def rand_storage(rng, shape, dtype, scale=1.0):
    """float32 values that are exact in the storage type."""
    x = (rng.standard_normal(shape) * scale).astype(np.float32)
    return wl.round_to_bf16(x) if dtype == "bf16" else x


def to_dev(torch, x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


GEMM_CASES = [
    # dtype, m, in, rows per segment, n_split
    ("fp32", 16, 256, (256, 256, 256), 1),      # tiny QKV
    ("fp32", 16, 256, (688, 688), 1),           # tiny gate/up: ragged 32-row blocks
    ("fp32", 16, 688, (256,), 1),               # tiny down: ragged K (688 = 10.75 iterations)
    ("fp32", 1, 688, (256,), 2),
    ("fp32", 33, 512, (96,), 2),
    ("bf16", 60, 4096, (1024, 256, 256), 4),    # GQA-style QKV, two token blocks
    ("bf16", 1, 4096, (512,), 4),               # plain decoding row
    ("bf16", 10, 11008, (128,), 8),             # draft frontier, long K, uneven slabs per split
    ("bf16", 64, 1280, (100,), 1),              # ragged rows, odd slab count
    ("bf16", 60, 256, (1000,), 1),              # one slab only
    ("bf16", 100, 2048, (160,), 2),             # four token blocks (tree-shape sweep sizes)
    ("bf16", 200, 1024, (96, 40), 2),           # two 128-row tiles (prefill), ragged second tile, two segments
    ("bf16", 512, 768, (300,), 1),              # four full tiles, ragged rows
    ("fp32", 129, 256, (64,), 1),               # second tile of a single row
]


@pytest.mark.parametrize("dtype,m,k,rows,n_split", GEMM_CASES)
def test_gemm_matches_matmul(env, dtype, m, k, rows, n_split):
    torch, P = env
    rng = np.random.default_rng(case_seed(dtype, m, k, rows))
    x = rand_storage(rng, (m, k), dtype)
    ws = [rand_storage(rng, (r, k), dtype, 0.05) for r in rows]
    part = P.spec_k_gemm(to_dev(torch, x, dtype), [to_dev(torch, w, dtype) for w in ws], n_split)
    torch.cuda.synchronize()
    got = part.cpu().numpy().astype(np.float64).sum(axis=0)
    want = x.astype(np.float64) @ np.concatenate(ws).astype(np.float64).T
    assert not np.isnan(got).any()
    tol = 2e-5 * np.sqrt(k) * 0.05 * (1 if dtype == "fp32" else 4)
    assert np.abs(got - want).max() < tol


@pytest.mark.parametrize("dtype,m,k,rows", [("fp32", 16, 256, 688), ("bf16", 60, 4096, 1100), ("bf16", 1, 1280, 64), ("bf16", 200, 768, 300),
                                            ("bf16", 40, 256, 77), ("fp32", 33, 128, 77), ("bf16", 60, 512, 15), ("bf16", 130, 256, 45)])
def test_gemm_swiglu_epilogue_matches_oracle(env, dtype, m, k, rows):
    """Gate and up projections with SwiGLU applied inside the launch: silu(x.wg) * (x.wu) against fp64, ragged 16-column
    blocks, one row, two 128-row tiles (the prefill form), an odd number of columns (no paired stores) and fewer columns
    than one block.  bf16 storage rounds the result once (relative 2^-9)."""
    torch, P = env
    rng = np.random.default_rng(case_seed("swiglu", dtype, m, k, rows))
    x = rand_storage(rng, (m, k), dtype)
    wg, wu = rand_storage(rng, (rows, k), dtype, 0.05), rand_storage(rng, (rows, k), dtype, 0.05)
    act = P.spec_k_gemm_swiglu(to_dev(torch, x, dtype), to_dev(torch, wg, dtype), to_dev(torch, wu, dtype))
    torch.cuda.synchronize()
    got = act.float().cpu().numpy().astype(np.float64)
    g = x.astype(np.float64) @ wg.astype(np.float64).T
    u = x.astype(np.float64) @ wu.astype(np.float64).T
    want = g / (1.0 + np.exp(-g)) * u
    assert not np.isnan(got).any()
    tol = 1e-5 * np.sqrt(k) + (2.0 ** -8 * np.abs(want) if dtype == "bf16" else 0.0)
    assert (np.abs(got - want) <= tol).all()


def expected_packed(rows_of_block, n_blocks, k_elems, esz, src_bytes_of_row):
    """The packed layout written out from its definition: tiles of 32 rows x 256 bytes of k, tiles of a block consecutive
    along k, piece (j, lane) of a tile at byte j*1024 + lane*16 = row lane%32, k-bytes (lane/32)*128 + j*16 .. +16 of the
    tile; zero beyond the matrix.  rows_of_block(b, c) -> source row or None; src_bytes_of_row(r) -> the row as bytes."""
    row_bytes = k_elems * esz
    n_it = (row_bytes + 255) // 256
    out = np.zeros((n_blocks, n_it, 8, 64, 16), dtype=np.uint8)
    for b in range(n_blocks):
        for c in range(32):
            r = rows_of_block(b, c)
            if r is None:
                continue
            src = np.zeros(n_it * 256, dtype=np.uint8)
            src[:row_bytes] = src_bytes_of_row(r)
            t = src.reshape(n_it, 2, 8, 16)                      # [tile][half g][piece j][16 bytes]
            for g in range(2):
                out[b, :, :, g * 32 + c, :] = t[:, g]
    return out.reshape(-1)


@pytest.mark.parametrize("dtype,rows,k", [("bf16", 77, 200), ("fp32", 45, 100), ("bf16", 64, 256)])
def test_packed_layouts_match_their_definition(env, dtype, rows, k):
    """spec_pack_weight and spec_pack_gate_up against the layout the header defines, byte for byte: ragged rows, ragged
    k, zero padding; gate/up: block b = gate rows 16b..16b+15 then up rows 16b..16b+15."""
    torch, P = env
    rng = np.random.default_rng(case_seed("pack", dtype, rows, k))
    esz = 2 if dtype == "bf16" else 4
    w, u = rand_storage(rng, (rows, k), dtype), rand_storage(rng, (rows, k), dtype)
    dw, du = to_dev(torch, w, dtype), to_dev(torch, u, dtype)
    raw = lambda t: t.contiguous().view(torch.uint8).cpu().numpy().reshape(rows, k * esz)
    bw, bu = raw(dw), raw(du)
    got = P.spec_pack_weight(dw)
    nb = (rows + 31) // 32
    want = expected_packed(lambda b, c: b * 32 + c if b * 32 + c < rows else None, nb, k, esz, lambda r: bw[r])
    assert got.numel() == want.size == P.spec_packed_bytes(1 if dtype == "bf16" else 0, rows, k)
    assert np.array_equal(got.cpu().numpy(), want)
    got = P.spec_pack_gate_up(dw, du)
    nb = (rows + 15) // 16

    def src_row(b, c):
        r = b * 16 + (c & 15)
        return (r if c < 16 else rows + r) if r < rows else None
    both = np.concatenate([bw, bu])
    want = expected_packed(src_row, nb, k, esz, lambda r: both[r])
    assert got.numel() == want.size
    assert np.array_equal(got.cpu().numpy(), want)
    assert P.spec_packed_bytes(1, 32, 12) == 0 and P.binding.lib.spec_packed_gate_up_bytes(0, 32, 6) == 0      # k not a whole 16-byte piece


def test_gemm_row_is_independent_of_batch(env):
    """A row computed alone (plain decoding) is bit-identical to the same row inside a 60-row tree."""
    torch, P = env
    rng = np.random.default_rng(3)
    x = to_dev(torch, rand_storage(rng, (60, 2048), "bf16"), "bf16")
    w = to_dev(torch, rand_storage(rng, (320, 2048), "bf16", 0.05), "bf16")
    full = P.spec_k_gemm(x, [w], 2)
    for i in (0, 17, 31, 32, 59):
        one = P.spec_k_gemm(x[i:i + 1].contiguous(), [w], 2)
        assert torch.equal(one[:, 0], full[:, i])
    ten = P.spec_k_gemm(x[5:15].contiguous(), [w], 2)
    assert torch.equal(ten, full[:, 5:15])


def make_tree(rng, rows, max_depth):
    par = np.full(rows, -1, np.int32)
    dep = np.zeros(rows, np.int32)
    for j in range(1, rows):
        cand = [p for p in range(j) if dep[p] < max_depth]
        par[j] = cand[int(rng.integers(len(cand)))]
        dep[j] = dep[par[j]] + 1
    anc = np.zeros((rows, 16), np.int32)
    for j in range(rows):
        a, q = j, dep[j]
        while a >= 0:
            anc[j, q] = a
            a, q = par[a], q - 1
    return par, dep, anc


def attention_error_ok(got, want, dtype, v_max):
    """got, want: arrays of the same shape.  fp32 storage: 1e-5.  bf16 storage: keys and values are exact, queries and
    probabilities enter the matrix cores as bf16 hi + lo pairs (relative 2^-16), sums are fp32, and the output is
    rounded to bf16 (relative 2^-9 of the element), so per element |err| <= 2^-8 |want| + 2^-12 max|v| and over the
    whole output rms(err) <= 2^-9 rms(want) + 1e-4.  With outputs of 0.03 .. 0.07 (averages over hundreds of
    unit-variance values) this is a few 1e-4: a dropped block of keys changes the output by several 1e-3."""
    err = np.abs(got - want)
    if dtype == "fp32":
        return err.max() < 1e-5
    per_elem = (err <= 2.0 ** -8 * np.abs(want) + 2.0 ** -12 * v_max).all()
    rms_ok = np.sqrt((err ** 2).mean()) <= 2.0 ** -9 * np.sqrt((want ** 2).mean()) + 1e-4
    return bool(per_elem and rms_ok)


ATTN_CASES = [
    # dtype, hq, hkv, hd, base, rows, tree?, query scale
    ("fp32", 4, 4, 64, 32, 16, True),
    ("fp32", 4, 2, 64, 0, 7, True),
    ("fp32", 8, 1, 128, 65, 16, True),
    ("fp32", 4, 4, 64, 250, 16, True),          # rows straddle the 256-position part boundary
    ("fp32", 4, 4, 64, 0, 64, False),           # prefill chunk from an empty cache
    ("bf16", 8, 8, 128, 511, 60, True),
    ("bf16", 8, 2, 128, 700, 60, True),
    ("bf16", 8, 1, 128, 63, 1, True),           # a single row (plain decoding)
    ("bf16", 4, 4, 128, 192, 64, False),        # chain crossing a part boundary
    ("fp32", 2, 1, 64, 1010, 24, True),         # rows straddle position 1024, where the parts become 256 keys long
    ("fp32", 2, 2, 64, 1500, 8, True),          # several of the longer parts, the last one ragged (vector path)
    ("bf16", 4, 2, 128, 1290, 40, True),        # the same on the matrix-core path
    ("bf16", 4, 2, 128, 1290, 40, True, 6.0),   # peaked scores: a few keys carry the row, outputs of order one
    ("bf16", 8, 1, 128, 2600, 12, True),        # 8 query heads per kv head (the 70B head layout), several far parts
    ("bf16", 2, 2, 64, 1100, 33, True, 6.0),    # head dim 64 on the matrix-core path
]


@pytest.mark.parametrize("case", ATTN_CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_attention_matches_oracle(env, case):
    torch, P = env
    dtype, hq, hkv, hd, base, rows, is_tree = case[:7]
    q_scale = case[7] if len(case) > 7 else 1.0
    rng = np.random.default_rng(case_seed(*case))
    slots = base + rows
    q = rand_storage(rng, (rows, hq * hd), dtype, q_scale)
    kc = rand_storage(rng, (slots, hkv * hd), dtype)
    vc = rand_storage(rng, (slots, hkv * hd), dtype)
    if is_tree:
        par, dep, anc = make_tree(rng, rows, 6)
    else:
        dep, anc = np.arange(rows, dtype=np.int32), None
    out = P.spec_k_attention(to_dev(torch, q, "fp32"), to_dev(torch, kc, dtype), to_dev(torch, vc, dtype), base,
                             torch.from_numpy(dep).cuda(), None if anc is None else torch.from_numpy(anc).cuda(), hq, hkv, hd)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().reshape(rows, hq, hd).astype(np.float64)
    g = hq // hkv
    k3, v3 = kc.reshape(slots, hkv, hd).astype(np.float64), vc.reshape(slots, hkv, hd).astype(np.float64)
    q3 = q.reshape(rows, hq, hd).astype(np.float64)
    want = np.zeros_like(got)
    for i in range(rows):
        vis = list(range(base)) + ([base + a for a in anc[i, :dep[i] + 1]] if is_tree else list(range(base, base + i + 1)))
        for h in range(hq):
            want[i, h] = attention_row(q3[i, h], k3[vis, h // g], v3[vis, h // g])
    assert attention_error_ok(got, want, dtype, np.abs(vc).max())


def test_attention_tree_row_equals_compacted_chain_row(env):
    """Bit-exactness by construction: a tree row gives the same bits as the same query over a cache in
    which its path has been moved to consecutive slots (what plain decoding sees after compaction)."""
    torch, P = env
    rng = np.random.default_rng(9)
    hq, hkv, hd, base, rows = 8, 2, 128, 300, 24
    par, dep, anc = make_tree(rng, rows, 5)
    q = to_dev(torch, rand_storage(rng, (rows, hq * hd), "bf16"), "fp32")
    kc = to_dev(torch, rand_storage(rng, (base + rows, hkv * hd), "bf16"), "bf16")
    vc = to_dev(torch, rand_storage(rng, (base + rows, hkv * hd), "bf16"), "bf16")
    tree_out = P.spec_k_attention(q, kc, vc, base, torch.from_numpy(dep).cuda(), torch.from_numpy(anc).cuda(), hq, hkv, hd)
    for i in (0, 5, rows - 1):
        path = [base + a for a in anc[i, :dep[i] + 1]]
        kc2, vc2 = kc.clone(), vc.clone()
        for d_, s in enumerate(path):
            kc2[base + d_], vc2[base + d_] = kc[s], vc[s]
        one = P.spec_k_attention(q[i:i + 1].contiguous(), kc2, vc2, base + int(dep[i]), torch.zeros(1, dtype=torch.int32).cuda(),
                                 None, hq, hkv, hd)
        assert torch.equal(one[0], tree_out[i])


@pytest.mark.parametrize("rows,vocab,k", [(1, 1024, 4), (4, 1024, 4), (10, 32000, 10), (10, 128256, 10), (3, 5000, 16), (16, 4097, 7)])
def test_topk_logprob_matches_oracle(env, rows, vocab, k):
    torch, P = env
    rng = np.random.default_rng(vocab + rows)
    logits = (rng.standard_normal((rows, vocab)) * 1.3).astype(np.float32)
    logits[0, 7] = logits[0, 900] = logits[0].max() + 1.0          # a tie for first place: lower index wins
    if rows > 1:
        logits[-1, vocab - 1] = logits[-1].max() + 2.0             # the last (ragged-slice) entry wins
    tok, lp = P.spec_k_topk_logprob(torch.from_numpy(logits).cuda(), k)
    torch.cuda.synchronize()
    tok, lp = tok.cpu().numpy(), lp.cpu().numpy()
    want_lp = log_softmax(logits.astype(np.float64))
    for r in range(rows):
        want = top_k(logits[r], k)
        assert list(tok[r]) == list(want)
        assert np.abs(lp[r] - want_lp[r, want]).max() < 5e-6
    assert tok[0, 0] == 7 and tok[0, 1] == 900 and (rows == 1 or tok[-1, 0] == vocab - 1)


@pytest.mark.parametrize("name,rows,k,n_split", [("70b-down", 8192, 28672, 4), ("70b-gateup-slice", 4096, 8192, 1), ("13b-qkv-slice", 5120, 5120, 2)])
def test_gemm_large_shapes_sampled_against_oracle(env, name, rows, k, n_split):
    """Matrix shapes of the largest configurations, M = 60: sampled output columns against fp64 dot products."""
    torch, P = env
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    x = (torch.randn(60, k, device="cuda", generator=g)).to(torch.bfloat16)
    w = (torch.randn(rows, k, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    got = P.spec_k_gemm(x, [w], n_split).sum(dim=0).cpu().numpy().astype(np.float64)
    cols = [0, 1, 31, 32, rows // 2 + 5, rows - 33, rows - 1]
    xs = x.float().cpu().numpy().astype(np.float64)
    for c in cols:
        want = xs @ w[c].float().cpu().numpy().astype(np.float64)
        assert np.abs(got[:, c] - want).max() < 2e-3


@pytest.mark.parametrize("q_scale", [1.0, 6.0], ids=["flat", "peaked"])
def test_attention_long_context_matches_oracle(env, q_scale):
    """Long-KV verify of the LLaMA3-8B configuration: 4100 cached keys (eight 128-key parts and thirteen 256-key parts
    on the matrix cores), GQA 4:1, sampled rows and heads; near-uniform and peaked score distributions."""
    torch, P = env
    rng = np.random.default_rng(77)
    hq, hkv, hd, base, rows = 8, 2, 128, 4100, 60
    par, dep, anc = make_tree(rng, rows, 6)
    q = rand_storage(rng, (rows, hq * hd), "bf16", q_scale)
    kc = rand_storage(rng, (base + rows, hkv * hd), "bf16")
    vc = rand_storage(rng, (base + rows, hkv * hd), "bf16")
    out = P.spec_k_attention(to_dev(torch, q, "fp32"), to_dev(torch, kc, "bf16"), to_dev(torch, vc, "bf16"), base,
                             torch.from_numpy(dep).cuda(), torch.from_numpy(anc).cuda(), hq, hkv, hd)
    got_all = out.float().cpu().numpy().reshape(rows, hq, hd).astype(np.float64)
    k3, v3 = kc.reshape(-1, hkv, hd).astype(np.float64), vc.reshape(-1, hkv, hd).astype(np.float64)
    q3 = q.reshape(rows, hq, hd).astype(np.float64)
    got, want = [], []
    for i in (0, 1, 17, 40, 59):
        vis = list(range(base)) + [base + a for a in anc[i, :dep[i] + 1]]
        for h in (0, 3, 4, 7):
            want.append(attention_row(q3[i, h], k3[vis, h // 4], v3[vis, h // 4]))
            got.append(got_all[i, h])
    assert attention_error_ok(np.array(got), np.array(want), "bf16", np.abs(vc).max())
