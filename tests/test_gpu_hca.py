"""GPU parity of the training attention of harmonized context alignment (spec_hca_attention, through the
C ABI) against oracle/hca.py on the same seeded inputs.

Tolerance (bf16 storage, inputs exact in bf16).  The kernel accumulates in fp32; what it rounds is each
probability (to bf16, relative 2^-9, before the value product) and the output (to bf16, relative 2^-9).
With out = sum p v and sum p = 1 both errors are at most 2^-9 max|v| each, so |error| <= 2^-8 max|v| holds
for every element; the typical error is far below (the roundings are independent), which the rms bound checks."""
import numpy as np
import pytest

import workload as wl
from oracle import hca

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2408_15766_amd as P
    assert torch.cuda.is_available()
    return torch, P


def run_gpu(torch, P, q, ks, vs):
    dev = lambda x: torch.from_numpy(x).cuda().to(torch.bfloat16)
    out = P.spec_hca_attention(dev(q), [dev(k) for k in ks], [dev(v) for v in vs])
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)


def check(got, want, vs, heads=None):
    if heads is not None:
        got, want = got[..., heads, :], want[..., heads, :]
    assert np.isfinite(got).all()
    vmax = max(float(np.abs(v).max()) for v in vs)
    err = np.abs(got - want)
    assert err.max() <= 2.0 ** -8 * vmax, f"max error {err.max():.4g} (bound {2.0 ** -8 * vmax:.4g})"
    rms = float(np.sqrt((err ** 2).mean()))
    assert rms <= 2.0 ** -9 * float(np.sqrt((want ** 2).mean())) + 1e-4, f"rms error {rms:.4g}"


CASES = [
    # n_streams, batch, seq, hq, hkv, hd
    (1, 1, 37, 2, 2, 128),        # plain causal, one ragged tile
    (2, 2, 130, 4, 2, 128),       # second tile of two queries, two batches, grouped heads
    (3, 1, 300, 4, 4, 128),       # the paper's three steps; three tiles, ragged tail
    (3, 2, 257, 8, 2, 64),        # head dim 64, four heads per kv head
    (4, 1, 64, 2, 1, 128),        # exactly one key block
    (5, 1, 5, 1, 1, 64),          # sequence shorter than the band is wide
    (8, 1, 200, 2, 2, 128),       # the most streams the entry point takes
    (3, 1, 1, 1, 1, 128),         # a single position
    (2, 3, 129, 6, 3, 128),       # kv groups not a multiple of 8, one query in the last tile
    (3, 1, 700, 4, 4, 128),       # six tiles, ragged tail
    (2, 2, 513, 8, 2, 64),        # head dim 64, one query in the last tile
    (8, 1, 600, 2, 1, 64),        # the widest band over several tiles
    (1, 1, 1000, 2, 2, 128),      # plain causal, longer
]


@pytest.mark.parametrize("n_streams,batch,seq,hq,hkv,hd", CASES)
def test_hca_attention_matches_oracle(env, n_streams, batch, seq, hq, hkv, hd):
    torch, P = env
    q, ks, vs = wl.make_hca_streams(11, n_streams, batch, seq, hq, hkv, hd)
    got = run_gpu(torch, P, q, ks, vs)
    for b in range(batch):
        want = hca.hca_attention(q[b].astype(np.float64), [k[b].astype(np.float64) for k in ks],
                                 [v[b].astype(np.float64) for v in vs])
        check(got[b], want, vs)


def test_hca_attention_peaked_scores(env):
    # wide score range: the running maximum moves from block to block and the rescaling path runs
    torch, P = env
    q, ks, vs = wl.make_hca_streams(12, 3, 1, 400, 2, 2, 128, q_scale=6.0)
    got = run_gpu(torch, P, q, ks, vs)
    want = hca.hca_attention(q[0].astype(np.float64), [k[0].astype(np.float64) for k in ks], [v[0].astype(np.float64) for v in vs])
    check(got[0], want, vs)


def test_hca_attention_near_target_streams(env):
    # draft streams that sit near the target's (the realistic case): a wrong stream choice would hide in a loose
    # tolerance, so this case is compared against the independent-stream bound as well
    torch, P = env
    q, ks, vs = wl.make_hca_streams(13, 3, 1, 200, 4, 2, 128, drift=0.3)
    got = run_gpu(torch, P, q, ks, vs)
    want = hca.hca_attention(q[0].astype(np.float64), [k[0].astype(np.float64) for k in ks], [v[0].astype(np.float64) for v in vs])
    check(got[0], want, vs)


@pytest.mark.parametrize("name,hq,hkv", [("llama2-7b draft layer", 32, 32), ("llama3-70b draft layer", 64, 8)])
def test_hca_attention_full_size_sampled_heads(env, name, hq, hkv):
    # the benchmark's launch: batch 2 (appendix, Training Overhead), 2048 positions, three streams.
    # The oracle computes three sampled heads per batch element.
    torch, P = env
    q, ks, vs = wl.make_hca_streams(14, 3, 2, 2048, hq, hkv, 128)
    got = run_gpu(torch, P, q, ks, vs)
    heads = [0, hq // 2 + 1, hq - 1]
    for b in range(2):
        want = hca.hca_attention(q[b].astype(np.float64), [k[b].astype(np.float64) for k in ks],
                                 [v[b].astype(np.float64) for v in vs], heads=heads)
        check(got[b], want, vs, heads=heads)


def test_hca_attention_rejects_bad_arguments(env):
    torch, P = env
    q, ks, vs = wl.make_hca_streams(15, 2, 1, 8, 2, 2, 128)
    dev = lambda x: torch.from_numpy(x).cuda().to(torch.bfloat16)
    dq, dks, dvs = dev(q), [dev(k) for k in ks], [dev(v) for v in vs]
    with pytest.raises(P.SpecError):
        P.spec_hca_attention(dq, dks * 5, dvs * 5)                       # ten streams
    with pytest.raises(P.SpecError):
        P.spec_hca_attention(dq[..., :96].contiguous(), [k[..., :96].contiguous() for k in dks],
                             [v[..., :96].contiguous() for v in dvs])    # head dim 96
    with pytest.raises(P.SpecError):
        P.spec_hca_attention(dev(np.zeros((1, 8, 3, 128), np.float32)), dks, dvs)   # 3 query heads over 2 kv heads
    torch.cuda.synchronize()
