"""Seeded synthetic inputs for the speculative-decoding hot path.

This module holds NO arithmetic of the method: only the shapes of the five
benchmark configurations, and seeded generators for weights and prompts.  It is
the one module that both the CPU oracle's callers and the HIP path's callers
read, so that both sides see the same bits.

The paper evaluates on trained LLaMA2-Chat 7B/13B and LLaMA3-Instruct 8B/70B
with trained draft heads on three public benchmarks (Sec. 4.1, Experimental
Setup).  None of those are available offline; the generators below stand in
for them with random-init weights N(0, 0.02) of the same shapes, norm weights 1,
and uniform-random prompt tokens.  Only the shapes are taken from the paper:
batch 1, a 60-token / depth-6 dynamic tree (Sec. 4.1, Implementation), T in
{0, 1}.
"""
from __future__ import annotations

import dataclasses
import hashlib
from typing import Dict, Iterator, List, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class Shape:
    """LLaMA-style decoder shape plus the draft-tree knobs of one configuration."""
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float
    dtype: str              # "fp32" | "bf16": storage type of weights/activations
    prompt_len: int
    tree_depth: int         # D: draft forwards per cycle (Drafting Hyper-Parameters appendix)
    tree_topk: int          # K
    tree_total: int         # N: rows of the verify forward, root included
    temperature: float
    gen_tokens: int
    rms_eps: float = 1e-5
    seed: int = 0

    def with_(self, **kw) -> "Shape":
        return dataclasses.replace(self, **kw)

    @property
    def d_q(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.head_dim


TINY = Shape("tiny", 2, 256, 4, 4, 64, 688, 1024, 1e4, "fp32", 32, 3, 4, 16, 0.0, 64)
LLAMA2_7B = Shape("llama2-7b", 32, 4096, 32, 32, 128, 11008, 32000, 1e4, "bf16", 512, 6, 10, 60, 0.0, 256)
LLAMA2_13B = Shape("llama2-13b", 40, 5120, 40, 40, 128, 13824, 32000, 1e4, "bf16", 512, 6, 10, 60, 1.0, 256)
LLAMA3_8B = Shape("llama3-8b", 32, 4096, 32, 8, 128, 14336, 128256, 5e5, "bf16", 4096, 6, 10, 60, 0.0, 512)
LLAMA3_70B = Shape("llama3-70b", 80, 8192, 64, 8, 128, 28672, 128256, 5e5, "bf16", 1024, 6, 10, 60, 0.0, 256)

CONFIGS: List[Shape] = [TINY, LLAMA2_7B, LLAMA2_13B, LLAMA3_8B, LLAMA3_70B]
BY_NAME: Dict[str, Shape] = {c.name: c for c in CONFIGS}

LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def tensor_specs(shape: Shape) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, dims, kind) for every tensor of target + draft, kind in {"normal", "ones"}.

    Projection matrices are stored row-major [out, in].
    """
    d, f, v = shape.d_model, shape.d_ffn, shape.vocab

    def layer(prefix: str):
        return [
            (prefix + "attn_norm", (d,), "ones"),
            (prefix + "wq", (shape.d_q, d), "normal"),
            (prefix + "wk", (shape.d_kv, d), "normal"),
            (prefix + "wv", (shape.d_kv, d), "normal"),
            (prefix + "wo", (d, shape.d_q), "normal"),
            (prefix + "ffn_norm", (d,), "ones"),
            (prefix + "w_gate", (f, d), "normal"),
            (prefix + "w_up", (f, d), "normal"),
            (prefix + "w_down", (d, f), "normal"),
        ]

    specs = [("embed", (v, d), "normal"), ("lm_head", (v, d), "normal"), ("final_norm", (d,), "ones")]
    for i in range(shape.n_layers):
        specs += layer(f"layers.{i}.")
    specs += [("draft.fc", (d, 2 * d), "normal")]
    specs += layer("draft.")
    return specs


def tensor_seed(run_seed: int, name: str) -> int:
    h = hashlib.sha256(f"{run_seed}:{name}".encode()).digest()
    return int.from_bytes(h[:8], "little")


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _draw(shape: Shape, name: str, dims, std: float) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=tensor_seed(shape.seed, name)))
    w = rng.standard_normal(dims, dtype=np.float32) * np.float32(std)
    return round_to_bf16(w) if shape.dtype == "bf16" else w


def make_weights(shape: Shape, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Host weights as float32 arrays.  For bf16 configs every value is bf16-representable.
    Each tensor has its own seeded stream, so tensors are drawn in parallel threads."""
    from concurrent.futures import ThreadPoolExecutor
    import os
    specs = tensor_specs(shape)
    out: Dict[str, np.ndarray] = {n: np.ones(d, dtype=np.float32) for n, d, k in specs if k == "ones"}
    todo = [(n, d) for n, d, k in specs if k == "normal"]
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        for (n, _), w in zip(todo, ex.map(lambda nd: _draw(shape, nd[0], nd[1], std), todo)):
            out[n] = w
    return {n: out[n] for n, _, _ in specs}


def make_prompt(shape: Shape, length: int | None = None) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=tensor_seed(shape.seed, "prompt")))
    n = shape.prompt_len if length is None else length
    return rng.integers(0, shape.vocab, size=n, dtype=np.int64).astype(np.int32)


def iter_device_weights(shape: Shape, device: str = "cuda", std: float = 0.02) -> Iterator[Tuple[str, "object"]]:
    """Yield (name, torch tensor on `device`) generated on the device, for sizes
    too large to draw on the host (the 70B shape is ~141 GB in bf16).  Values
    differ from make_weights(); use only where no oracle comparison on the same
    weights is made, or copy the tensors back to the host for the oracle.
    """
    import torch

    tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
    for name, dims, kind in tensor_specs(shape):
        if kind == "ones":
            yield name, torch.ones(dims, dtype=tdt, device=device)
            continue
        g = torch.Generator(device=device)
        g.manual_seed(tensor_seed(shape.seed, name) & 0x7FFFFFFFFFFFFFFF)
        rows = dims[0]
        t = torch.empty(dims, dtype=tdt, device=device)
        step = max(1, (1 << 26) // max(1, int(np.prod(dims[1:]))))
        for r0 in range(0, rows, step):
            r1 = min(rows, r0 + step)
            blk = torch.randn((r1 - r0,) + tuple(dims[1:]), dtype=torch.float32, device=device, generator=g)
            t[r0:r1] = (blk * std).to(tdt)
        yield name, t


def algorithmic_bytes(shape: Shape) -> Dict[str, float]:
    """Bytes each forward must read once from HBM (weights only), by shape arithmetic."""
    esz = 2 if shape.dtype == "bf16" else 4
    d, f, v = shape.d_model, shape.d_ffn, shape.vocab
    layer = (shape.d_q * d + 2 * shape.d_kv * d + d * shape.d_q + 3 * f * d) * esz
    head = v * d * esz
    fc = 2 * d * d * esz
    kv_per_token = 2 * shape.d_kv * esz * shape.n_layers
    return {
        "layer": layer, "lm_head": head, "draft_fc": fc,
        "verify_weights": shape.n_layers * layer + head,
        "draft_forward": layer + fc + head,
        "kv_bytes_per_token": kv_per_token,
    }


def graft_continuation(token, parent, depth, n_nodes: int, continuation) -> int:
    """Edits a drafted tree (host arrays: token, parent, depth; node 0 = root, parents precede children) so that it
    contains `continuation` as a root-to-node path: follows an existing child where there is one, otherwise re-parents
    a leaf that is not on the path, and overwrites the tokens on the path.  Returns the length of the grafted path.
    Input preparation only (teacher-forced trees for tests and for the benchmark's acceptance-length mode): it does
    none of the method's arithmetic."""
    n = int(n_nodes)
    par = parent[:n]
    cur, on_path, done = 0, {0}, 0
    for tok in continuation:
        kids = np.nonzero(par == cur)[0]
        if kids.size:
            c = int(kids[0])
        else:
            n_kids = np.bincount(par[1:], minlength=n)
            leaves = [int(j) for j in np.nonzero(n_kids == 0)[0] if j > cur and int(j) not in on_path]
            if not leaves:
                break
            c = leaves[0]
            par[c] = cur
        token[c] = int(tok)
        cur = c
        on_path.add(c)
        done += 1
    for j in range(1, n):
        depth[j] = depth[par[j]] + 1
    return done


def make_hca_streams(seed: int, n_streams: int, batch: int, seq: int, hq: int, hkv: int, hd: int, q_scale: float = 1.0,
                     drift: float | None = None):
    """Seeded inputs of the training attention: queries [batch, seq, hq, hd] and, per stream, keys and values
    [batch, seq, hkv, hd]; float32 arrays whose values are exact in bf16.  Unit-variance normal entries, so
    q.k / sqrt(hd) has unit variance (q_scale widens it).  drift = None draws every stream independently (the
    demanding case for a test: a wrong stream changes the output by O(1)); a number makes stream m equal to
    stream 0 plus m * drift of independent noise, the way draft features sit near the target's.
    Input preparation only: none of the method's arithmetic."""
    rng = np.random.Generator(np.random.Philox(key=tensor_seed(seed, f"hca:{n_streams}:{batch}:{seq}:{hq}:{hkv}:{hd}")))
    q = round_to_bf16(rng.standard_normal((batch, seq, hq, hd), dtype=np.float32) * np.float32(q_scale))
    ks, vs = [], []
    for m in range(n_streams):
        k = rng.standard_normal((batch, seq, hkv, hd), dtype=np.float32)
        v = rng.standard_normal((batch, seq, hkv, hd), dtype=np.float32)
        if drift is not None and m > 0:
            k = ks[0] + np.float32(m * drift) * k
            v = vs[0] + np.float32(m * drift) * v
        ks.append(round_to_bf16(k))
        vs.append(round_to_bf16(v))
    return q, ks, vs


def make_distill_inputs(seed: int, rows: int, d: int, vocab: int, dtype: str, drift: float = 0.5, tie_halves: bool = False,
                        logit_std: float = 3.0):
    """Seeded inputs of the distillation loss: target features [rows, d] (unit-variance normal, as after a final
    norm), draft features = target + drift * independent noise (a draft model's estimate), LM head [vocab, d]
    normal with the spread that gives logits of standard deviation logit_std (a peaked next-token distribution:
    the best token of 32000 holds a few percent to tens of percent of the mass, the way a language model's does);
    float32 arrays, exact in bf16 when dtype == "bf16".  tie_halves repeats the first half of the LM head in the
    second half, so that every logit occurs twice (exact ties).
    Input preparation only: none of the method's arithmetic."""
    rng = np.random.Generator(np.random.Philox(key=tensor_seed(seed, f"distill:{rows}:{d}:{vocab}:{dtype}")))
    ft = rng.standard_normal((rows, d), dtype=np.float32)
    fd = ft + np.float32(drift) * rng.standard_normal((rows, d), dtype=np.float32)
    w = rng.standard_normal((vocab, d), dtype=np.float32) * np.float32(logit_std / np.sqrt(d))
    if tie_halves:
        w[vocab // 2: 2 * (vocab // 2)] = w[: vocab // 2]
    if dtype == "bf16":
        ft, fd, w = round_to_bf16(ft), round_to_bf16(fd), round_to_bf16(w)
    return ft, fd, w
