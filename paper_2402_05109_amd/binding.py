"""ctypes binding of libhydra.so: same names as include/hydra.h, argument
marshalling only.  PyTorch supplies device memory and the current stream; every
step of the decoding path runs inside the library's HIP kernels.

There is no fallback: if the shared library is missing the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhydra.so")

HYDRA_F32, HYDRA_BF16 = 0, 1
HYDRA_OK = 0
E_INVALID_ARG, E_SHAPE, E_CAPACITY, E_UNSUPPORTED, E_HIP, E_STATE = -1, -2, -3, -4, -5, -6

(W_EMBED, W_LM_HEAD, W_FINAL_NORM, W_ATTN_NORM, W_WQ, W_WK, W_WV, W_WO, W_FFN_NORM, W_GATE, W_UP, W_DOWN,
 W_HEAD_W1, W_HEAD_B1, W_HEAD_WL, W_HEAD_BL, W_HEAD_WOUT) = range(17)

EXPORTS = ["hydra_create", "hydra_destroy", "hydra_last_error", "hydra_weights_bytes", "hydra_bind_weights",
           "hydra_load_tensor", "hydra_workspace_bytes", "hydra_read_flags", "hydra_draft_tree",
           "tree_verify_forward", "tree_attention", "accept_greedy", "accept_typical", "accept_typical_static", "kv_compact", "hydra_prefix_attention", "hydra_tree_depth",
           "hydra_kv_write", "hydra_kv_read", "hydra_profile_begin", "hydra_profile_end", "hydra_layer_kernel_info"]


class ModelDesc(C.Structure):
    _fields_ = [("d", C.c_int32), ("n_layers", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn", C.c_int32), ("vocab", C.c_int32), ("dtype", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float), ("page_size", C.c_int32), ("max_pos", C.c_int32)]


class HeadsDesc(C.Structure):
    _fields_ = [("n_draft_heads", C.c_int32), ("mlp_layers", C.c_int32), ("include_root_embedding", C.c_int32),
                ("medusa", C.c_int32)]


class TreeDesc(C.Structure):
    _fields_ = [("T", C.c_int32), ("parent", C.POINTER(C.c_int32))]


class KVDesc(C.Structure):
    _fields_ = [("k_pages", C.c_void_p), ("v_pages", C.c_void_p), ("page_table", C.c_void_p),
                ("n_pages", C.c_int32), ("max_pages", C.c_int32), ("seq_len_hint", C.c_int32)]


class HydraError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libhydra error {code}: {msg}")
        self.code = code


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2402_05109_amd.build` "
                          "(there is no CPU or PyTorch fallback for the Hydra hot path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    lib.hydra_last_error.restype = C.c_char_p
    lib.hydra_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(HeadsDesc), C.POINTER(TreeDesc), i32, C.POINTER(vp)]
    lib.hydra_destroy.argtypes = [vp]
    lib.hydra_weights_bytes.argtypes = [vp]; lib.hydra_weights_bytes.restype = sz
    lib.hydra_bind_weights.argtypes = [vp, vp, vp, i32]
    lib.hydra_load_tensor.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.hydra_workspace_bytes.argtypes = [vp, i32]; lib.hydra_workspace_bytes.restype = sz
    lib.hydra_read_flags.argtypes = [vp, vp, C.POINTER(C.c_int32)]
    lib.hydra_draft_tree.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    lib.tree_verify_forward.argtypes = [vp, vp, i32, vp, vp, vp, C.POINTER(KVDesc), vp, vp, vp, vp]
    lib.tree_attention.argtypes = [vp, vp, i32, i32, vp, vp, vp, C.POINTER(KVDesc), vp]
    lib.accept_greedy.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.accept_typical.argtypes = [vp, vp, i32, vp, vp, vp, C.c_float, C.c_float, C.c_float, vp, vp, vp, vp, vp]
    lib.accept_typical_static.argtypes = [vp, vp, i32, vp, vp, C.c_float, C.c_float, C.c_float, vp, vp, vp, vp, vp]
    lib.kv_compact.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, C.POINTER(KVDesc), vp, vp, vp, vp]
    lib.hydra_prefix_attention.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, vp, C.POINTER(KVDesc), vp]
    lib.hydra_tree_depth.argtypes = [vp]
    lib.hydra_kv_write.argtypes = [vp, vp, i32, i32, C.POINTER(KVDesc), i32, i32, vp]
    lib.hydra_kv_read.argtypes = [vp, vp, i32, i32, C.POINTER(KVDesc), i32, i32, vp]
    lib.hydra_profile_begin.argtypes = [vp]
    lib.hydra_layer_kernel_info.argtypes = [vp, i32, C.POINTER(C.c_int64)]
    lib.hydra_profile_end.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    return lib


_lib = _load()


def lib() -> C.CDLL:
    return _lib


def last_error() -> str:
    return _lib.hydra_last_error().decode()


def _check(rc: int) -> None:
    if rc != HYDRA_OK:
        raise HydraError(rc, last_error())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor], dtype: torch.dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of {dtype}, got {t.dtype} on {t.device}")
    return t.data_ptr()


class KV:
    """Caller-owned paged KV cache (see hydra_kv in the header)."""

    def __init__(self, k_pages: torch.Tensor, v_pages: torch.Tensor, page_table: torch.Tensor, n_pages: int,
                 seq_len_hint: int = 0):
        assert page_table.dtype == torch.int32 and page_table.is_cuda and page_table.is_contiguous()
        self.k_pages, self.v_pages, self.page_table = k_pages, v_pages, page_table
        self.n_pages, self.max_pages = int(n_pages), int(page_table.shape[-1])
        self.seq_len_hint = int(seq_len_hint)

    def desc(self) -> KVDesc:
        return KVDesc(self.k_pages.data_ptr(), self.v_pages.data_ptr(), self.page_table.data_ptr(),
                      self.n_pages, self.max_pages, self.seq_len_hint)


class Hydra:
    """One library context = one (model, heads, tree) triple."""

    def __init__(self, *, d, n_layers, n_heads, head_dim, ffn, vocab, dtype, rms_eps=1e-6, rope_theta=10000.0,
                 max_pos=8192, n_draft_heads=0, mlp_layers=1, include_root_embedding=1, medusa=0,
                 parent: Sequence[int] = (-1,), max_batch=1, page_size=16):
        self.model = ModelDesc(d, n_layers, n_heads, head_dim, ffn, vocab, dtype, rms_eps, rope_theta, page_size, max_pos)
        self.heads = HeadsDesc(n_draft_heads, mlp_layers, include_root_embedding, medusa)
        self.T = len(parent)
        arr = (C.c_int32 * self.T)(*[int(p) for p in parent])
        tree = TreeDesc(self.T, arr)
        h = C.c_void_p()
        _check(_lib.hydra_create(C.byref(self.model), C.byref(self.heads), C.byref(tree), int(max_batch), C.byref(h)))
        self._h = h
        self.max_batch = max_batch
        self.depth = _lib.hydra_tree_depth(self._h)
        self.torch_dtype = torch.bfloat16 if dtype == HYDRA_BF16 else torch.float32

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.hydra_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    # ---- weights / workspace
    def weights_bytes(self) -> int:
        return _lib.hydra_weights_bytes(self._h)

    def bind_weights(self, arena: torch.Tensor, table_slot: int = 0) -> None:
        _check(_lib.hydra_bind_weights(self._h, _stream(), _ptr(arena, torch.uint8, "arena"), int(table_slot)))
        self._arena = arena

    def load_tensor(self, kind: int, index: int, sub: int, src: torch.Tensor) -> None:
        _check(_lib.hydra_load_tensor(self._h, _stream(), kind, index, sub, _ptr(src, self.torch_dtype, "src")))

    def workspace_bytes(self, B: int) -> int:
        return _lib.hydra_workspace_bytes(self._h, int(B))

    def read_flags(self) -> int:
        out = C.c_int32(0)
        _check(_lib.hydra_read_flags(self._h, _stream(), C.byref(out)))
        return out.value

    # ---- hot path
    def hydra_draft_tree(self, B, ws, h_last, root, tree_tokens) -> None:
        _check(_lib.hydra_draft_tree(self._h, _stream(), B, _ptr(ws, torch.uint8, "ws"),
                                     _ptr(h_last, torch.float32, "h_last"), _ptr(root, torch.int32, "root"),
                                     _ptr(tree_tokens, torch.int32, "tree_tokens")))

    def tree_verify_forward(self, B, ws, tree_tokens, seq_len, kv: KV, hidden, argmax, margin=None, logits=None) -> None:
        d = kv.desc()
        _check(_lib.tree_verify_forward(self._h, _stream(), B, _ptr(ws, torch.uint8, "ws"),
                                        _ptr(tree_tokens, torch.int32, "tree_tokens"),
                                        _ptr(seq_len, torch.int32, "seq_len"), C.byref(d),
                                        _ptr(hidden, torch.float32, "hidden"), _ptr(argmax, torch.int32, "argmax"),
                                        _ptr(margin, torch.float32, "margin"), _ptr(logits, torch.float32, "logits")))

    def tree_attention(self, B, layer, ws, q, seq_len, kv: KV, out) -> None:
        d = kv.desc()
        _check(_lib.tree_attention(self._h, _stream(), B, layer, _ptr(ws, torch.uint8, "ws"),
                                   _ptr(q, torch.float32, "q"), _ptr(seq_len, torch.int32, "seq_len"), C.byref(d),
                                   _ptr(out, torch.float32, "out")))

    def accept_greedy(self, B, tree_tokens, argmax, n_acc, path, next_root, last_node) -> None:
        _check(_lib.accept_greedy(self._h, _stream(), B, _ptr(tree_tokens, torch.int32, "tree_tokens"),
                                  _ptr(argmax, torch.int32, "argmax"), _ptr(n_acc, torch.int32, "n_acc"),
                                  _ptr(path, torch.int32, "path"), _ptr(next_root, torch.int32, "next_root"),
                                  _ptr(last_node, torch.int32, "last_node")))

    def accept_typical(self, B, ws, tree_tokens, logits, tau, eps, alpha, u, n_acc, path, next_root, last_node) -> None:
        _check(_lib.accept_typical(self._h, _stream(), B, _ptr(ws, torch.uint8, "ws"), _ptr(tree_tokens, torch.int32, "tree_tokens"),
                                   _ptr(logits, torch.float32, "logits"), float(tau), float(eps), float(alpha),
                                   _ptr(u, torch.float32, "u"), _ptr(n_acc, torch.int32, "n_acc"),
                                   _ptr(path, torch.int32, "path"), _ptr(next_root, torch.int32, "next_root"),
                                   _ptr(last_node, torch.int32, "last_node")))

    def accept_typical_static(self, B, tree_tokens, logits, tau, eps, alpha, u, n_acc, path, next_root, last_node) -> None:
        _check(_lib.accept_typical_static(self._h, _stream(), B, _ptr(tree_tokens, torch.int32, "tree_tokens"),
                                          _ptr(logits, torch.float32, "logits"), float(tau), float(eps), float(alpha),
                                          _ptr(u, torch.float32, "u"), _ptr(n_acc, torch.int32, "n_acc"),
                                          _ptr(path, torch.int32, "path"), _ptr(next_root, torch.int32, "next_root"),
                                          _ptr(last_node, torch.int32, "last_node")))

    def kv_compact(self, B, n_acc, path, next_root, last_node, hidden, kv: KV, seq_len, h_last, root, kv_index=None) -> None:
        d = kv.desc()
        _check(_lib.kv_compact(self._h, _stream(), B, _ptr(n_acc, torch.int32, "n_acc"), _ptr(path, torch.int32, "path"),
                               _ptr(next_root, torch.int32, "next_root"), _ptr(last_node, torch.int32, "last_node"),
                               _ptr(hidden, torch.float32, "hidden"), C.byref(d), _ptr(seq_len, torch.int32, "seq_len"),
                               _ptr(h_last, torch.float32, "h_last"), _ptr(root, torch.int32, "root"),
                               _ptr(kv_index, torch.int32, "kv_index")))

    def hydra_prefix_attention(self, B, ws, hidden, T_src, path, n_acc, seq_len, kv: KV, h_out) -> None:
        d = kv.desc()
        _check(_lib.hydra_prefix_attention(self._h, _stream(), B, _ptr(ws, torch.uint8, "workspace"),
                                           _ptr(hidden, torch.float32, "hidden"), T_src, _ptr(path, torch.int32, "path"),
                                           _ptr(n_acc, torch.int32, "n_acc"), _ptr(seq_len, torch.int32, "seq_len"),
                                           C.byref(d), _ptr(h_out, torch.float32, "h_out")))

    # ---- harness helpers
    def kv_write(self, B, layer, kv: KV, first_slot, n_slots, plain) -> None:
        d = kv.desc()
        _check(_lib.hydra_kv_write(self._h, _stream(), B, layer, C.byref(d), first_slot, n_slots,
                                   _ptr(plain, torch.float32, "kv_plain")))

    def kv_read(self, B, layer, kv: KV, first_slot, n_slots, plain) -> None:
        d = kv.desc()
        _check(_lib.hydra_kv_read(self._h, _stream(), B, layer, C.byref(d), first_slot, n_slots,
                                  _ptr(plain, torch.float32, "kv_plain")))

    def layer_kernel_info(self, B: int):
        info = (C.c_int64 * 4)()
        _check(_lib.hydra_layer_kernel_info(self._h, B, info))
        return list(info)

    def profile_begin(self) -> None:
        _check(_lib.hydra_profile_begin(self._h))

    def profile_end(self):
        n, ms, by = C.c_int64(0), C.c_double(0), C.c_double(0)
        _check(_lib.hydra_profile_end(self._h, C.byref(n), C.byref(ms), C.byref(by)))
        return n.value, ms.value, by.value
