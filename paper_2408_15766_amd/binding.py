"""ctypes binding of libspec.so: same names as the C ABI, argument marshalling only.

torch is used for device memory (weights, the workspace) and for the current HIP stream; no
arithmetic of the decode path happens in Python.  There is no CPU fallback: if the library has not
been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import dataclasses
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libspec.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_2408_15766_amd/build.py` "
                      "(there is no fallback path)")
lib = C.CDLL(_LIB_PATH)

SPEC_OK, SPEC_EINVAL, SPEC_ESTATE, SPEC_ECAP, SPEC_EHIP = 0, -1, -2, -3, -4
SPEC_MAX_DEPTH, SPEC_MAX_TOPK, SPEC_MAX_NODES = 15, 16, 128
LAYER_FIELDS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate_up", "w_down")


class SpecError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libspec error {code}: {msg}")
        self.code = code


class spec_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32), ("max_seq", C.c_int32),
                ("tree_depth", C.c_int32), ("tree_topk", C.c_int32), ("tree_total", C.c_int32),
                ("temperature", C.c_float), ("seed", C.c_uint64), ("device", C.c_int32), ("stream", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_uint64)]


class spec_layer_weights(C.Structure):
    _fields_ = [(f, C.c_void_p) for f in LAYER_FIELDS]


class spec_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("layers", C.POINTER(spec_layer_weights)), ("draft_fc", C.c_void_p), ("draft_layer", spec_layer_weights)]


class spec_tree(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("token", C.POINTER(C.c_int32)), ("parent", C.POINTER(C.c_int32)),
                ("depth", C.POINTER(C.c_int32)), ("score", C.POINTER(C.c_float))]


_i32p, _f32p = C.POINTER(C.c_int32), C.POINTER(C.c_float)
lib.spec_workspace_bytes.restype = C.c_uint64
lib.spec_workspace_bytes.argtypes = [C.POINTER(spec_config)]
lib.spec_create.argtypes = [C.POINTER(spec_config), C.POINTER(spec_weights), C.POINTER(C.c_void_p)]
lib.spec_prefill.argtypes = [C.c_void_p, _i32p, C.c_int32, _i32p]
lib.spec_draft_tree.argtypes = [C.c_void_p, C.POINTER(spec_tree)]
lib.spec_verify.argtypes = [C.c_void_p, C.POINTER(spec_tree)]
lib.spec_accept.argtypes = [C.c_void_p, C.POINTER(spec_tree), _i32p, _i32p]
lib.spec_destroy.argtypes = [C.c_void_p]
lib.spec_destroy.restype = None
lib.spec_committed.argtypes = [C.c_void_p]
lib.spec_get_logits.restype = C.c_int64
lib.spec_get_logits.argtypes = [C.c_void_p, _f32p, C.c_int64]
lib.spec_get_features.restype = C.c_int64
lib.spec_get_features.argtypes = [C.c_void_p, _f32p, C.c_int64]
lib.spec_get_kv.restype = C.c_int64
lib.spec_get_kv.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _f32p, _f32p, C.c_int64]
lib.spec_set_profile.argtypes = [C.c_void_p, C.c_int32]
lib.spec_set_graphs.argtypes = [C.c_void_p, C.c_int32]
lib.spec_get_profile.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
lib.spec_static_tree_bytes.restype = C.c_uint64
lib.spec_static_tree_bytes.argtypes = [C.POINTER(spec_config), C.c_int32, _i32p, _i32p, C.c_int32]
lib.spec_set_static_tree.argtypes = [C.c_void_p, C.c_int32, _i32p, _i32p, C.c_int32, C.c_void_p, C.c_uint64]
lib.spec_last_error.restype = C.c_char_p
lib.spec_last_error.argtypes = [C.c_void_p]
lib.spec_packed_bytes.restype = C.c_uint64
lib.spec_packed_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
lib.spec_pack_weight.argtypes = [C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
lib.spec_packed_gate_up_bytes.restype = C.c_uint64
lib.spec_packed_gate_up_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
lib.spec_pack_gate_up.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
lib.spec_k_gemm.argtypes = [C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                            C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
lib.spec_k_gemm_swiglu.argtypes = [C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
lib.spec_k_attention.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                 C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
lib.spec_k_topk_logprob.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_void_p]
lib.spec_k_topk_logprob_static.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
lib.spec_k_accept_qratio.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_uint64,
                                     C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
lib.spec_k_sample_children.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_int32, C.c_uint64, C.c_uint32, C.c_uint32, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p]
lib.spec_hca_attention.argtypes = [C.c_int32, C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int32, C.c_int32,
                                   C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
lib.spec_topk_loss_scratch_bytes.restype = C.c_uint64
lib.spec_topk_loss_scratch_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
lib.spec_topk_loss.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                               C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]


@dataclasses.dataclass
class Tree:
    """Host-side flattened draft tree (numpy views of the arrays handed to the C ABI)."""
    token: np.ndarray
    parent: np.ndarray
    depth: np.ndarray
    score: np.ndarray
    n_nodes: int

    @staticmethod
    def empty(capacity: int) -> "Tree":
        return Tree(np.zeros(capacity, np.int32), np.zeros(capacity, np.int32), np.zeros(capacity, np.int32),
                    np.zeros(capacity, np.float32), 0)

    def as_c(self) -> spec_tree:
        for a in (self.token, self.parent, self.depth, self.score):
            assert a.flags["C_CONTIGUOUS"]
        return spec_tree(self.n_nodes, self.token.ctypes.data_as(_i32p), self.parent.ctypes.data_as(_i32p),
                         self.depth.ctypes.data_as(_i32p), self.score.ctypes.data_as(_f32p))


def _check(ctx, rc: int):
    if rc < 0:
        raise SpecError(rc, (lib.spec_last_error(ctx) or b"").decode())
    return rc


def spec_last_error(ctx) -> str:
    return (lib.spec_last_error(ctx) or b"").decode()


def spec_workspace_bytes(cfg: spec_config) -> int:
    return int(lib.spec_workspace_bytes(C.byref(cfg)))


def spec_create(cfg: spec_config, w: spec_weights):
    out = C.c_void_p()
    _check(None, lib.spec_create(C.byref(cfg), C.byref(w), C.byref(out)))
    return out


def spec_destroy(ctx) -> None:
    lib.spec_destroy(ctx)


def spec_committed(ctx) -> int:
    return int(lib.spec_committed(ctx))


def spec_prefill(ctx, prompt: np.ndarray) -> int:
    p = np.ascontiguousarray(prompt, dtype=np.int32)
    first = C.c_int32()
    _check(ctx, lib.spec_prefill(ctx, p.ctypes.data_as(_i32p), len(p), C.byref(first)))
    return int(first.value)


def spec_draft_tree(ctx, tree: Tree) -> Tree:
    t = tree.as_c()
    _check(ctx, lib.spec_draft_tree(ctx, C.byref(t)))
    tree.n_nodes = int(t.n_nodes)
    return tree


def spec_verify(ctx, tree: Tree) -> None:
    t = tree.as_c()
    _check(ctx, lib.spec_verify(ctx, C.byref(t)))


def spec_accept(ctx, tree: Tree) -> List[int]:
    t = tree.as_c()
    out = (C.c_int32 * (SPEC_MAX_DEPTH + 1))()
    n = C.c_int32()
    _check(ctx, lib.spec_accept(ctx, C.byref(t), out, C.byref(n)))
    return [int(out[i]) for i in range(n.value)]


def spec_get_logits(ctx, n_nodes: int, vocab: int) -> np.ndarray:
    buf = np.empty((n_nodes, vocab), dtype=np.float32)
    _check(ctx, lib.spec_get_logits(ctx, buf.ctypes.data_as(_f32p), buf.size))
    return buf


def spec_get_features(ctx, n_nodes: int, d: int) -> np.ndarray:
    buf = np.empty((n_nodes, d), dtype=np.float32)
    _check(ctx, lib.spec_get_features(ctx, buf.ctypes.data_as(_f32p), buf.size))
    return buf


def spec_get_kv(ctx, which: int, layer: int, n_rows: int, d_kv: int):
    k = np.empty((n_rows, d_kv), dtype=np.float32)
    v = np.empty((n_rows, d_kv), dtype=np.float32)
    _check(ctx, lib.spec_get_kv(ctx, which, layer, n_rows, k.ctypes.data_as(_f32p), v.ctypes.data_as(_f32p), k.size))
    return k, v


def spec_set_graphs(ctx, enable: bool) -> None:
    _check(ctx, lib.spec_set_graphs(ctx, 1 if enable else 0))


def spec_set_profile(ctx, level: int) -> None:
    _check(ctx, lib.spec_set_profile(ctx, level))


def spec_get_profile(ctx):
    ms = (C.c_double * 8)()
    cnt = (C.c_int64 * 8)()
    _check(ctx, lib.spec_get_profile(ctx, ms, cnt))
    return [float(x) for x in ms], [int(x) for x in cnt]


def _stream_ptr(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def spec_packed_bytes(dtype: int, rows: int, cols: int) -> int:
    return int(lib.spec_packed_bytes(dtype, rows, cols))


def spec_pack_weight(w):
    """Row-major torch matrix [rows, in] on the device -> packed copy (uint8 tensor that remembers its shape)."""
    import torch
    assert w.is_contiguous() and w.dim() == 2
    dtype = 1 if w.dtype == torch.bfloat16 else 0
    n = spec_packed_bytes(dtype, w.shape[0], w.shape[1])
    if n == 0:
        raise SpecError(SPEC_EINVAL, f"cannot pack a {tuple(w.shape)} {w.dtype} matrix")
    dst = torch.empty(n, dtype=torch.uint8, device=w.device)
    rc = lib.spec_pack_weight(dtype, w.data_ptr(), w.shape[0], w.shape[1], dst.data_ptr(), _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_pack_weight")
    dst.logical_shape = tuple(w.shape)
    return dst


def spec_pack_gate_up(w_gate, w_up):
    """Row-major torch matrices [rows, in] on the device -> the one packed gate/up matrix (uint8 tensor)."""
    import torch
    assert w_gate.is_contiguous() and w_up.is_contiguous() and w_gate.dim() == 2 and w_gate.shape == w_up.shape and w_gate.dtype == w_up.dtype
    dtype = 1 if w_gate.dtype == torch.bfloat16 else 0
    n = int(lib.spec_packed_gate_up_bytes(dtype, w_gate.shape[0], w_gate.shape[1]))
    if n == 0:
        raise SpecError(SPEC_EINVAL, f"cannot pack {tuple(w_gate.shape)} {w_gate.dtype} gate/up matrices")
    dst = torch.empty(n, dtype=torch.uint8, device=w_gate.device)
    rc = lib.spec_pack_gate_up(dtype, w_gate.data_ptr(), w_up.data_ptr(), w_gate.shape[0], w_gate.shape[1], dst.data_ptr(), _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_pack_gate_up")
    dst.logical_shape = tuple(w_gate.shape)
    return dst


PACKED_TENSORS = ("wq", "wk", "wv", "wo", "w_down", "lm_head", "fc")


def is_packed_name(name: str) -> bool:
    return name.rsplit(".", 1)[-1] in PACKED_TENSORS


def spec_k_gemm(x, ws: Sequence, n_split: int, m: Optional[int] = None):
    """x: torch [m, in]; ws: 1..3 row-major torch weight matrices [rows, in] (packed here, per call: test use).
    Returns fp32 torch [n_split, m, cols]."""
    import torch
    dtype = 1 if x.dtype == torch.bfloat16 else 0
    m = x.shape[0] if m is None else m
    rows = [w.shape[0] for w in ws] + [0] * (3 - len(ws))
    packed = [spec_pack_weight(w.contiguous()) for w in ws]
    ptrs = [C.c_void_p(w.data_ptr()) for w in packed] + [None] * (3 - len(ws))
    cols = sum(rows)
    part = torch.full((n_split, m, cols), float("nan"), dtype=torch.float32, device=x.device)
    rc = lib.spec_k_gemm(dtype, x.data_ptr(), x.stride(0), m, x.shape[1], ptrs[0], rows[0], ptrs[1], rows[1], ptrs[2], rows[2],
                         part.data_ptr(), cols, m, n_split, _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_k_gemm")
    return part


def spec_k_gemm_swiglu(x, w_gate, w_up, packed=None):
    """x: torch [m, in]; w_gate, w_up: row-major torch [rows, in] (packed here, per call: test use) -> act [m, rows].
    packed: optional packed gate/up matrix from spec_pack_gate_up, to keep packing out of a timed loop."""
    import torch
    dtype = 1 if x.dtype == torch.bfloat16 else 0
    pgu = packed if packed is not None else spec_pack_gate_up(w_gate.contiguous(), w_up.contiguous())
    rows = pgu.logical_shape[0]
    act = torch.full((x.shape[0], rows), float("nan"), dtype=x.dtype, device=x.device)
    rc = lib.spec_k_gemm_swiglu(dtype, x.data_ptr(), x.stride(0), x.shape[0], x.shape[1], pgu.data_ptr(), rows, act.data_ptr(), _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_k_gemm_swiglu")
    return act


def spec_k_attention(q, kcache, vcache, base: int, depth, anc, hq: int, hkv: int, hd: int):
    """q: fp32 [rows, hq*hd]; caches [slots, hkv*hd] in the storage type; depth int32 [rows]; anc int32 [rows,16] or None.
    Returns [rows, hq*hd] in the storage type."""
    import torch
    assert q.dtype == torch.float32
    dtype = 1 if kcache.dtype == torch.bfloat16 else 0
    rows = q.shape[0]
    max_depth = int(depth.max().item())
    max_parts = (base + max_depth) // 128 + 2
    scratch = torch.empty(rows * hq * max_parts * (hd + 2), dtype=torch.float32, device=q.device)
    out = torch.empty(q.shape, dtype=kcache.dtype, device=q.device)
    rc = lib.spec_k_attention(dtype, q.data_ptr(), kcache.data_ptr(), vcache.data_ptr(), rows, hq, hkv, hd, base,
                              depth.data_ptr(), None if anc is None else anc.data_ptr(), max_depth, scratch.data_ptr(),
                              max_parts, out.data_ptr(), _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_k_attention")
    return out


def spec_k_topk_logprob(logits, k: int):
    import torch
    rows, vocab = logits.shape
    ns = (vocab + 4095) // 4096
    sf = torch.empty(16 * ns * 18, dtype=torch.float32, device=logits.device)
    si = torch.empty(16 * ns * 16, dtype=torch.int32, device=logits.device)
    tok = torch.zeros((rows, 16), dtype=torch.int32, device=logits.device)
    lp = torch.zeros((rows, 16), dtype=torch.float32, device=logits.device)
    rc = lib.spec_k_topk_logprob(logits.data_ptr(), rows, vocab, k, sf.data_ptr(), si.data_ptr(), tok.data_ptr(), lp.data_ptr(),
                                 _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_k_topk_logprob")
    return tok[:, :k], lp[:, :k]


def spec_k_topk_logprob_static(logits, k: int, top_tok=None, top_lp=None):
    """The same call without scratch arguments (the library's static scratch).  top_tok / top_lp: optional preallocated
    int32 / fp32 [rows, 16] outputs, so that a caller can keep the call itself free of allocations."""
    import torch
    rows, vocab = logits.shape
    tok = torch.zeros((rows, 16), dtype=torch.int32, device=logits.device) if top_tok is None else top_tok
    lp = torch.zeros((rows, 16), dtype=torch.float32, device=logits.device) if top_lp is None else top_lp
    rc = lib.spec_k_topk_logprob_static(logits.data_ptr(), rows, vocab, k, tok.data_ptr(), lp.data_ptr(), _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_k_topk_logprob_static")
    return tok[:, :k], lp[:, :k]


def spec_k_accept_qratio(p_logits, q_logits, tree_tok, tree_par, temperature: float, seed: int, cycle: int):
    """p_logits, q_logits: fp32 torch [n_nodes, vocab]; tree_tok, tree_par: int32 torch [n_nodes].
    Returns (accepted nodes, tokens): tokens = the accepted tokens followed by the next token."""
    import torch
    n, vocab = p_logits.shape
    assert q_logits.shape == p_logits.shape and p_logits.dtype == torch.float32 and q_logits.dtype == torch.float32
    assert p_logits.is_contiguous() and q_logits.is_contiguous()
    work = torch.empty(vocab, dtype=torch.float32, device=p_logits.device)
    res = torch.zeros(33, dtype=torch.int32, device=p_logits.device)
    rc = lib.spec_k_accept_qratio(p_logits.data_ptr(), q_logits.data_ptr(), n, vocab, temperature, tree_tok.data_ptr(),
                                  tree_par.data_ptr(), seed, cycle, work.data_ptr(), res.data_ptr(), _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_k_accept_qratio")
    r = res.cpu().numpy()
    m = int(r[0])
    return [int(x) for x in r[2:2 + m]], [int(x) for x in r[17:18 + m]]


def spec_k_sample_children(logits, temperature: float, m: int, seed: int, cycle: int, node_stream: int):
    """logits: fp32 torch [vocab].  Returns the m sampled tokens in draw order."""
    import torch
    assert logits.dtype == torch.float32 and logits.dim() == 1 and logits.is_contiguous()
    out = torch.zeros(m, dtype=torch.int32, device=logits.device)
    vocab = logits.shape[0]
    ns = (vocab + 4095) // 4096
    sf = torch.empty(vocab + 16 * ns * 18 + 32, dtype=torch.float32, device=logits.device)
    si = torch.empty(16 * ns * 16 + 16, dtype=torch.int32, device=logits.device)
    rc = lib.spec_k_sample_children(logits.data_ptr(), vocab, temperature, m, seed, cycle, node_stream, sf.data_ptr(), si.data_ptr(),
                                    out.data_ptr(), _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_k_sample_children")
    return [int(x) for x in out.cpu().numpy()]


def spec_hca_attention(q, ks: Sequence, vs: Sequence, out=None):
    """q: bf16 torch [batch, seq, hq, hd]; ks[m], vs[m]: bf16 [batch, seq, hkv, hd], one pair per stream
    (stream 0 = target features, stream m = draft features of training step m).  Returns bf16 [batch, seq, hq, hd]."""
    import torch
    n = len(ks)
    assert len(vs) == n and q.dtype == torch.bfloat16 and q.is_contiguous()
    assert all(x.dtype == torch.bfloat16 and x.is_contiguous() and x.shape == ks[0].shape for x in list(ks) + list(vs))
    batch, seq, hq, hd = q.shape
    hkv = ks[0].shape[2]
    assert ks[0].shape == (batch, seq, hkv, hd)
    if out is None:
        out = torch.empty_like(q)
    kp = (C.c_void_p * n)(*[x.data_ptr() for x in ks])
    vp = (C.c_void_p * n)(*[x.data_ptr() for x in vs])
    rc = lib.spec_hca_attention(n, q.data_ptr(), kp, vp, batch, seq, hq, hkv, hd, out.data_ptr(), _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_hca_attention")
    return out


def spec_topk_loss_scratch_bytes(rows: int, vocab: int, k: int) -> int:
    return int(lib.spec_topk_loss_scratch_bytes(rows, vocab, k))


def spec_topk_loss(feat_target, feat_draft, lm_head_packed, k: int, scratch=None):
    """feat_target, feat_draft: torch [rows, d] (bf16 or fp32); lm_head_packed: the LM head after spec_pack_weight.
    Returns (loss_topk [rows], loss_ce [rows], loss_sum [2]) as fp32 torch tensors."""
    import torch
    assert feat_target.shape == feat_draft.shape and feat_target.dtype == feat_draft.dtype
    assert feat_target.is_contiguous() and feat_draft.is_contiguous()
    dtype = 1 if feat_target.dtype == torch.bfloat16 else 0
    rows, d = feat_target.shape
    vocab = lm_head_packed.logical_shape[0]
    n = spec_topk_loss_scratch_bytes(rows, vocab, k)
    if n == 0:
        raise SpecError(SPEC_EINVAL, f"spec_topk_loss: rows {rows}, vocab {vocab}, k {k} not supported")
    if scratch is None:
        scratch = torch.empty(n, dtype=torch.uint8, device=feat_target.device)
    topk = torch.empty(rows, dtype=torch.float32, device=feat_target.device)
    ce = torch.empty(rows, dtype=torch.float32, device=feat_target.device)
    tot = torch.empty(2, dtype=torch.float32, device=feat_target.device)
    rc = lib.spec_topk_loss(dtype, feat_target.data_ptr(), feat_draft.data_ptr(), rows, d, lm_head_packed.data_ptr(), vocab, k,
                            scratch.data_ptr(), scratch.numel(), topk.data_ptr(), ce.data_ptr(), tot.data_ptr(), _stream_ptr())
    if rc:
        raise SpecError(rc, "spec_topk_loss")
    return topk, ce, tot


def pack_weights(named_tensors, tap=None) -> Dict[str, "object"]:
    """(name, row-major device tensor) pairs -> dict with every projection matrix in the packed layout; a layer's
    w_gate and w_up (which must follow each other) become its w_gate_up.  Matrices are packed one at a time and the
    row-major original is dropped, so the peak extra memory is one matrix (two for gate/up).  tap(name, tensor), if
    given, sees every row-major tensor before it is packed."""
    out = {}
    gate = None
    for name, t in named_tensors:
        if tap is not None:
            tap(name, t)
        leaf = name.rsplit(".", 1)[-1]
        if leaf == "w_gate":
            gate = (name, t.contiguous())
        elif leaf == "w_up":
            assert gate is not None and gate[0][:-len("w_gate")] == name[:-len("w_up")], "w_up must follow its layer's w_gate"
            out[name[:-len("w_up")] + "w_gate_up"] = spec_pack_gate_up(gate[1], t.contiguous())
            gate = None
        else:
            out[name] = spec_pack_weight(t.contiguous()) if is_packed_name(name) else t.contiguous()
        del t
    assert gate is None, "w_gate without w_up"
    return out


def upload_weights(host: Dict[str, np.ndarray], dtype: str, device: str = "cuda") -> Dict[str, "object"]:
    """numpy float32 weights -> device tensors in the storage type, projections packed (plumbing only)."""
    import torch
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    return pack_weights((k, torch.from_numpy(np.ascontiguousarray(v)).to(device=device, dtype=tdt)) for k, v in host.items())


class Engine:
    """Owns the torch-allocated workspace and the weight pointer table of one libspec context."""

    def __init__(self, shape, weights: Dict[str, "object"], *, max_seq: Optional[int] = None, temperature: Optional[float] = None,
                 seed: int = 0, tree=None, device: int = 0, graphs: bool = True, workspace_fill: int = 0):
        import torch
        self.shape = shape
        # a stream of its own (default priority): graph capture is not possible on the default stream
        torch.cuda.synchronize(device)                  # weights were produced on torch's current stream
        self.stream = torch.cuda.Stream(device=device)
        self.weights = weights                         # keeps the tensors alive: the library borrows them
        depth, topk, total = tree if tree is not None else (shape.tree_depth, shape.tree_topk, shape.tree_total)
        self.total = total
        if max_seq is None:
            max_seq = shape.prompt_len + shape.gen_tokens + total + SPEC_MAX_DEPTH + 2
        cfg = spec_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                          shape.rope_theta, shape.rms_eps, 1 if shape.dtype == "bf16" else 0, max_seq, depth, topk, total,
                          shape.temperature if temperature is None else temperature, seed, device,
                          self.stream.cuda_stream, None, 0)
        nbytes = spec_workspace_bytes(cfg)
        if nbytes == 0:
            raise SpecError(SPEC_EINVAL, "invalid configuration")
        # the library initialises what it reads; `workspace_fill` lets a test hand over a dirty workspace
        self.workspace = torch.full((nbytes,), workspace_fill, dtype=torch.uint8, device=f"cuda:{device}")
        cfg.workspace = self.workspace.data_ptr()
        cfg.workspace_bytes = nbytes
        self.cfg = cfg

        def ptr(name):
            return C.c_void_p(weights[name].data_ptr())
        self._layers = (spec_layer_weights * shape.n_layers)()
        for l in range(shape.n_layers):
            for f in LAYER_FIELDS:
                setattr(self._layers[l], f, weights[f"layers.{l}.{f}"].data_ptr())
        w = spec_weights()
        w.embed, w.lm_head, w.final_norm, w.draft_fc = ptr("embed"), ptr("lm_head"), ptr("final_norm"), ptr("draft.fc")
        w.layers = C.cast(self._layers, C.POINTER(spec_layer_weights))
        for f in LAYER_FIELDS:
            setattr(w.draft_layer, f, weights[f"draft.{f}"].data_ptr())
        self._w = w
        torch.cuda.synchronize(device)                  # workspace fill done before the library's stream uses it
        self.ctx = spec_create(cfg, w)
        if not graphs:
            spec_set_graphs(self.ctx, False)
        self.tree = Tree.empty(max(total, 1))

    def close(self):
        if getattr(self, "ctx", None):
            spec_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_static_tree(self, parent, rank, sampled: bool = False) -> None:
        """Draft a fixed tree shape from now on (see spec_set_static_tree); parent = [] returns to the dynamic tree."""
        import torch
        par = np.ascontiguousarray(parent, dtype=np.int32)
        rk = np.ascontiguousarray(rank, dtype=np.int32)
        n = int(par.shape[0])
        if n == 0:
            _check(self.ctx, lib.spec_set_static_tree(self.ctx, 0, None, None, 0, None, 0))
            self._static_buffer = None
            return
        pp, rp = par.ctypes.data_as(_i32p), rk.ctypes.data_as(_i32p)
        nbytes = int(lib.spec_static_tree_bytes(C.byref(self.cfg), n, pp, rp, int(sampled)))
        buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.workspace.device)
        _check(self.ctx, lib.spec_set_static_tree(self.ctx, n, pp, rp, int(sampled), buf.data_ptr(), nbytes))
        self._static_buffer = buf                       # borrowed by the library

    # one-to-one with the C ABI
    def prefill(self, prompt) -> int:
        return spec_prefill(self.ctx, prompt)

    def draft_tree(self) -> Tree:
        return spec_draft_tree(self.ctx, self.tree)

    def verify(self, tree: Optional[Tree] = None) -> None:
        spec_verify(self.ctx, self.tree if tree is None else tree)

    def accept(self, tree: Optional[Tree] = None) -> List[int]:
        return spec_accept(self.ctx, self.tree if tree is None else tree)

    def logits(self, n_nodes: Optional[int] = None) -> np.ndarray:
        return spec_get_logits(self.ctx, self.tree.n_nodes if n_nodes is None else n_nodes, self.shape.vocab)

    def features(self, n_nodes: Optional[int] = None) -> np.ndarray:
        return spec_get_features(self.ctx, self.tree.n_nodes if n_nodes is None else n_nodes, self.shape.d_model)

    def kv(self, which: int, layer: int, n_rows: int):
        return spec_get_kv(self.ctx, which, layer, n_rows, self.shape.n_kv_heads * self.shape.head_dim)

    @property
    def committed(self) -> int:
        return spec_committed(self.ctx)

    def generate(self, prompt, gen: int, tree_hook=None, record: Optional[list] = None):
        """prefill + cycles until `gen` tokens; returns (tokens[:gen], emitted-per-cycle)."""
        out = [self.prefill(prompt)]
        taus = []
        while len(out) < gen:
            t = self.draft_tree()
            if tree_hook is not None:
                t = tree_hook(self, t)
            self.verify(t)
            if record is not None:
                record.append(dict(n=self.committed, tree=dataclasses.replace(
                    t, token=t.token[:t.n_nodes].copy(), parent=t.parent[:t.n_nodes].copy(), depth=t.depth[:t.n_nodes].copy(),
                    score=t.score[:t.n_nodes].copy()), logits=self.logits(t.n_nodes), feats=self.features(t.n_nodes)))
            emitted = self.accept(t)
            if record is not None:
                record[-1]["emitted"] = list(emitted)
            out += emitted
            taus.append(len(emitted))
        return out[:gen], taus
