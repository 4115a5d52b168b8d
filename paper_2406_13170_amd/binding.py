"""Thin ctypes binding of libamph.so: same names as include/amph.h, argument marshalling only.

Device buffers are torch tensors (PyTorch is used for device memory and streams, nothing else);
every step of the path runs in the library's HIP kernels.  Loading fails loudly when the shared
library has not been built: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libamph.so")

AMPH_OK, AMPH_EINVAL, AMPH_ESHAPE, AMPH_ETREE, AMPH_EHIP = 0, 1, 2, 3, 4
AMPH_F32, AMPH_BF16 = 0, 1
AMPH_DEV_SAL_OVERFLOW, AMPH_DEV_KV_OVERFLOW, AMPH_DEV_BAD_TOKEN = 1, 2, 4
KERNEL_KINDS = ["fc", "sal_qkv", "sal_attn", "sal_wo", "sal_gateup", "sal_down", "head_mlp", "aeb_qkv", "aeb_attn", "aeb_wo",
                "lm_head", "topk", "t_rmsnorm", "t_qkv", "verify", "t_wo", "t_gateup", "t_down", "t_lmhead"]
STATUS_NAMES = {0: "AMPH_OK", 1: "AMPH_EINVAL", 2: "AMPH_ESHAPE", 3: "AMPH_ETREE", 4: "AMPH_EHIP"}


class amph_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d_model", "n_heads", "head_dim", "d_ffn", "vocab", "K", "topk", "max_tree",
                                         "max_kv", "batch", "dtype")] + [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("n_stages", "aeb_layers", "lm_rank")]


class amph_layer_w(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("rms1", "wq", "wk", "wv", "wo", "rms2", "w_gate", "w_up", "w_down")]


class amph_layer_tiled(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("qkv", "wo", "gate_up", "down")]


AMPH_PACK_QKV, AMPH_PACK_WO, AMPH_PACK_GATEUP, AMPH_PACK_DOWN, AMPH_PACK_LMHEAD = range(5)


class amph_draft_w(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("fc", C.c_void_p * 2), ("sal", amph_layer_w * 2), ("mlp", C.c_void_p),
                ("pe", C.c_void_p), ("aeb_wq", C.c_void_p), ("aeb_wk", C.c_void_p), ("aeb_wv", C.c_void_p),
                ("aeb_wo", C.c_void_p), ("lm_head", C.c_void_p), ("aeb2_wq", C.c_void_p), ("aeb2_wk", C.c_void_p),
                ("aeb2_wv", C.c_void_p), ("aeb2_wo", C.c_void_p), ("lm_a", C.c_void_p), ("lm_b", C.c_void_p)]


EXPORTS = {
    "amph_create": (C.c_int, [C.POINTER(amph_config), C.POINTER(C.c_void_p)]),
    "amph_destroy": (None, [C.c_void_p]),
    "amph_set_stream": (C.c_int, [C.c_void_p, C.c_void_p]),
    "amph_workspace_bytes": (C.c_size_t, [C.c_void_p]),
    "amph_last_error": (C.c_char_p, [C.c_void_p]),
    "amph_device_status": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32)]),
    "amph_draft": (C.c_int, [C.c_void_p, C.POINTER(amph_draft_w), C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "amph_commit": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int] + [C.c_void_p] * 11),
    "amph_tree_create": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_void_p)]),
    "amph_tree_destroy": (None, [C.c_void_p]),
    "amph_tree_info": (C.c_int, [C.c_void_p, C.POINTER(C.c_int), C.POINTER(C.c_int)] + [C.POINTER(C.c_void_p)] * 5),
    "amph_tree_build": (C.c_int, [C.c_void_p] * 7),
    "amph_verify_attn": (C.c_int, [C.c_void_p] * 8),
    "amph_verify_attn_static": (C.c_int, [C.c_void_p] * 7),
    "amph_pack_kv": (C.c_int, [C.c_void_p] * 5 + [C.c_int]),
    "amph_unpack_kv": (C.c_int, [C.c_void_p] * 5 + [C.c_int]),
    "amph_accept": (C.c_int, [C.c_void_p] * 10),
    "amph_accept_typical": (C.c_int, [C.c_void_p] * 4 + [C.c_float] * 3 + [C.c_void_p] * 6),
    "amph_target_forward": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(amph_layer_w), C.POINTER(amph_layer_tiled), C.c_int]
                            + [C.c_void_p] * 13),
    "amph_tiled_bytes": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_size_t)]),
    "amph_pack_weights": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "amph_verify_kernel": (C.c_int, [C.c_void_p, C.c_int]),
    "amph_profile_kind": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int]),
    "amph_profile_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int)]),
    "amph_gemv": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int]),
    "amph_gemm": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
}

_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (python -c 'import __graft_entry__ as g; g.build()')."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (__graft_entry__.build()); there is no fallback")
        _lib = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(_lib, name)
            fn.restype = res
            fn.argtypes = args
    return _lib


class AmphError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} {detail}")
        self.status = status


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


class Tree:
    """amph_tree handle.  paths: sequences of top-k ranks (root implicit)."""

    def __init__(self, paths: Sequence[Sequence[int]], K: int):
        arr = np.full((len(paths), K), -1, dtype=np.int32)
        for i, p in enumerate(paths):
            p = [int(r) for r in p if r >= 0]
            if len(p) > K:
                raise AmphError(AMPH_ETREE, "amph_tree_create", "path longer than K")
            arr[i, :len(p)] = p
        self._arr = np.ascontiguousarray(arr)
        h = C.c_void_p()
        st = lib().amph_tree_create(self._arr.ctypes.data_as(C.c_void_p), len(paths), K, C.byref(h))
        if st != AMPH_OK:
            raise AmphError(st, "amph_tree_create")
        self.handle = h
        self.K = K
        T, nl = C.c_int(), C.c_int()
        ptrs = [C.c_void_p() for _ in range(5)]
        st = lib().amph_tree_info(h, C.byref(T), C.byref(nl), *[C.byref(p) for p in ptrs])
        if st != AMPH_OK:
            raise AmphError(st, "amph_tree_info")
        self.T, self.n_leaves = T.value, nl.value

        def view(p, ctype, n):
            return np.ctypeslib.as_array(C.cast(p, C.POINTER(ctype)), shape=(n,)).copy()
        self.parent = view(ptrs[0], C.c_int32, self.T)
        self.depth = view(ptrs[1], C.c_int32, self.T)
        self.rank = view(ptrs[2], C.c_int32, self.T)
        self.mask_bits = view(ptrs[3], C.c_uint64, self.T * 2).reshape(self.T, 2)
        self.retrieve = view(ptrs[4], C.c_int32, self.n_leaves * (K + 1)).reshape(self.n_leaves, K + 1)

    def mask_bool(self) -> np.ndarray:
        m = np.zeros((self.T, self.T), dtype=bool)
        for i in range(self.T):
            for j in range(self.T):
                m[i, j] = (int(self.mask_bits[i, j >> 6]) >> (j & 63)) & 1
        return m

    def close(self):
        if self.handle:
            lib().amph_tree_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Context:
    """amph_ctx handle plus the caller-owned workspace (a torch uint8 tensor on the device)."""

    def __init__(self, *, d_model, n_heads, head_dim, d_ffn, vocab, K, topk, max_tree, max_kv, batch, dtype,
                 rms_eps=1e-6, rope_theta=10000.0, n_stages=2, aeb_layers=1, lm_rank=0, device="cuda:0",
                 alloc_workspace=True):
        self.cfg = amph_config(d_model, n_heads, head_dim, d_ffn, vocab, K, topk, max_tree, max_kv, batch, dtype,
                               rms_eps, rope_theta, n_stages, aeb_layers, lm_rank)
        h = C.c_void_p()
        st = lib().amph_create(C.byref(self.cfg), C.byref(h))
        if st != AMPH_OK:
            raise AmphError(st, "amph_create")
        self.handle = h
        self.device = device
        self.workspace = None
        self._keep: List[object] = []
        if alloc_workspace:
            import torch
            self.workspace = torch.empty(self.workspace_bytes() + 256, dtype=torch.uint8, device=device)
            self.set_stream(torch.cuda.current_stream(torch.device(device)).cuda_stream)

    # -- plumbing
    def _check(self, st: int, where: str):
        if st != AMPH_OK:
            raise AmphError(st, where, lib().amph_last_error(self.handle).decode())

    def set_stream(self, stream_ptr: int):
        self._check(lib().amph_set_stream(self.handle, C.c_void_p(stream_ptr)), "amph_set_stream")

    def workspace_bytes(self) -> int:
        return int(lib().amph_workspace_bytes(self.handle))

    def device_status(self) -> int:
        bits = C.c_uint32()
        self._check(lib().amph_device_status(self.handle, C.byref(bits)), "amph_device_status")
        return bits.value

    def close(self):
        if self.handle:
            lib().amph_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights
    @staticmethod
    def layer_struct(lw: Dict[str, object]) -> amph_layer_w:
        return amph_layer_w(*[_ptr(lw[k]) for k in ("rms1", "wq", "wk", "wv", "wo", "rms2", "w_gate", "w_up", "w_down")])

    @staticmethod
    def draft_struct(dw: Dict[str, object]) -> amph_draft_w:
        s = amph_draft_w()
        s.embed = _ptr(dw["embed"])
        for i, (fc, sal) in enumerate(zip(dw["fc"], dw["sal"])):      # one entry each for the one-adaptation-layer variant
            s.fc[i], s.sal[i] = _ptr(fc), Context.layer_struct(sal)
        s.mlp, s.pe = _ptr(dw["mlp"]), _ptr(dw.get("pe"))
        s.aeb_wq, s.aeb_wk, s.aeb_wv, s.aeb_wo = (_ptr(dw[k]) for k in ("aeb_wq", "aeb_wk", "aeb_wv", "aeb_wo"))
        s.lm_head = _ptr(dw.get("lm_head"))
        s.aeb2_wq, s.aeb2_wk, s.aeb2_wv, s.aeb2_wo = (_ptr(dw.get(k)) for k in ("aeb2_wq", "aeb2_wk", "aeb2_wv", "aeb2_wo"))
        s.lm_a, s.lm_b = _ptr(dw.get("lm_a")), _ptr(dw.get("lm_b"))
        return s

    # -- the calls of include/amph.h
    def amph_draft(self, dw_struct: amph_draft_w, h_new, tok_new, sal_kv, sal_len, topk_idx, topk_val, logits=None, n_new=1,
                   n_valid=None):
        self._check(lib().amph_draft(self.handle, C.byref(dw_struct), _ptr(h_new), _ptr(tok_new), n_new, _ptr(n_valid),
                                     _ptr(sal_kv), _ptr(sal_len), _ptr(topk_idx), _ptr(topk_val), _ptr(logits),
                                     _ptr(self.workspace)), "amph_draft")

    def amph_commit(self, tree: Tree, n_layers, k_caches, v_caches, kv_len, accept_len, accept_path, next_tok=None,
                    tree_tok=None, hidden=None, h_new=None, tok_new=None, n_new=None):
        self._check(lib().amph_commit(self.handle, tree.handle, n_layers, _ptr(k_caches), _ptr(v_caches), _ptr(kv_len),
                                      _ptr(accept_len), _ptr(accept_path), _ptr(next_tok), _ptr(tree_tok), _ptr(hidden),
                                      _ptr(h_new), _ptr(tok_new), _ptr(n_new)), "amph_commit")

    def amph_tree_build(self, tree: Tree, root_tok, topk_idx, kv_len, tree_tok, tree_pos):
        self._check(lib().amph_tree_build(self.handle, tree.handle, _ptr(root_tok), _ptr(topk_idx), _ptr(kv_len),
                                          _ptr(tree_tok), _ptr(tree_pos)), "amph_tree_build")

    def amph_verify_attn(self, tree: Tree, q, k_cache, v_cache, kv_len, out):
        self._check(lib().amph_verify_attn(self.handle, tree.handle, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(kv_len),
                                           _ptr(out), _ptr(self.workspace)), "amph_verify_attn")

    def amph_verify_attn_static(self, tree: Tree, q, k_cache, v_cache, kv_len, out):
        self._check(lib().amph_verify_attn_static(self.handle, tree.handle, _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                                  _ptr(kv_len), _ptr(out)), "amph_verify_attn_static")

    def amph_pack_kv(self, k_rows, v_rows, k_tiled, v_tiled, n_caches: int):
        self._check(lib().amph_pack_kv(self.handle, _ptr(k_rows), _ptr(v_rows), _ptr(k_tiled), _ptr(v_tiled), n_caches),
                    "amph_pack_kv")

    def amph_unpack_kv(self, k_tiled, v_tiled, k_rows, v_rows, n_caches: int):
        self._check(lib().amph_unpack_kv(self.handle, _ptr(k_tiled), _ptr(v_tiled), _ptr(k_rows), _ptr(v_rows), n_caches),
                    "amph_unpack_kv")

    def amph_accept(self, tree: Tree, tree_tok, tgt_argmax, tgt_logits, accept_len, accept_path, next_tok, best_node):
        self._check(lib().amph_accept(self.handle, tree.handle, _ptr(tree_tok), _ptr(tgt_argmax), _ptr(tgt_logits),
                                      _ptr(accept_len), _ptr(accept_path), _ptr(next_tok), _ptr(best_node),
                                      _ptr(self.workspace)), "amph_accept")

    def amph_accept_typical(self, tree: Tree, tree_tok, tgt_logits, temperature, eps, delta, u, accept_len, accept_path,
                            next_tok, best_node):
        self._check(lib().amph_accept_typical(self.handle, tree.handle, _ptr(tree_tok), _ptr(tgt_logits),
                                              float(temperature), float(eps), float(delta), _ptr(u), _ptr(accept_len),
                                              _ptr(accept_path), _ptr(next_tok), _ptr(best_node), _ptr(self.workspace)),
                    "amph_accept_typical")

    def amph_target_forward(self, tree: Tree, layer_structs, embed, final_norm, lm_head, tree_tok, tree_pos, k_caches,
                            v_caches, kv_len, hidden_out, logits_out, tgt_argmax, tiled_structs=None, lm_head_tiled=None):
        n = len(layer_structs)
        arr = (amph_layer_w * max(n, 1))(*layer_structs)
        tarr = None
        if tiled_structs is not None:
            assert len(tiled_structs) == n
            tarr = (amph_layer_tiled * max(n, 1))(*tiled_structs)
        self._check(lib().amph_target_forward(self.handle, tree.handle, arr, tarr, n, _ptr(embed), _ptr(final_norm),
                                              _ptr(lm_head), _ptr(lm_head_tiled), _ptr(tree_tok), _ptr(tree_pos),
                                              _ptr(k_caches), _ptr(v_caches), _ptr(kv_len), _ptr(hidden_out),
                                              _ptr(logits_out), _ptr(tgt_argmax), _ptr(self.workspace)),
                    "amph_target_forward")

    def amph_tiled_bytes(self, role: int) -> int:
        n = C.c_size_t()
        self._check(lib().amph_tiled_bytes(self.handle, role, C.byref(n)), "amph_tiled_bytes")
        return n.value

    def amph_pack_weights(self, role: int, w0, w1, w2, dst):
        self._check(lib().amph_pack_weights(self.handle, role, _ptr(w0), _ptr(w1), _ptr(w2), _ptr(dst)), "amph_pack_weights")

    def amph_verify_kernel(self, kernel: int):
        self._check(lib().amph_verify_kernel(self.handle, kernel), "amph_verify_kernel")

    def amph_profile_kind(self, kind: int, max_launches: int = 4096, every: int = 1):
        self._check(lib().amph_profile_kind(self.handle, kind, max_launches, every), "amph_profile_kind")

    def amph_profile_read(self):
        ms, n = C.c_double(), C.c_int()
        self._check(lib().amph_profile_read(self.handle, C.byref(ms), C.byref(n)), "amph_profile_read")
        return ms.value, n.value

    def amph_gemv(self, x, W, y, M, N, Kd):
        self._check(lib().amph_gemv(self.handle, _ptr(x), _ptr(W), _ptr(y), M, N, Kd), "amph_gemv")

    def amph_gemm(self, x, W, y, M, N, Kd, split_k=0):
        self._check(lib().amph_gemm(self.handle, _ptr(x), _ptr(W), _ptr(y), M, N, Kd, split_k, _ptr(self.workspace)),
                    "amph_gemm")
