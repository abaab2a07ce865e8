"""ctypes binding of libmedusa_hip.so: same names as include/medusa.h, argument marshalling only.

Every step of the path runs in the library's HIP kernels.  PyTorch is used for device memory
(tensors own the buffers, `data_ptr()` is what crosses the boundary) and for the current
stream.  There is no fallback: if the library is missing or a call fails, an exception is
raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

# MEDUSA_LIB_PATH names another build of the same library (the host-sanitizer build the CPU tests use).
_LIB_PATH = os.environ.get("MEDUSA_LIB_PATH") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmedusa_hip.so")
_lib_handle = None

MEDUSA_F32, MEDUSA_BF16 = 0, 1
MEDUSA_GREEDY, MEDUSA_TYPICAL = 0, 1

EXPORTED_SYMBOLS = (
    "medusa_status_string", "medusa_tree_create_cartesian", "medusa_tree_create_nodes",
    "medusa_tree_create_optimized", "medusa_tree_destroy",
    "medusa_tree_query", "medusa_tree_tables", "medusa_heads", "medusa_topk_tree_workspace_bytes",
    "medusa_topk_tree", "tree_attention_workspace_bytes", "tree_attention", "tree_attention_static",
    "tree_attention_static_scratch_bytes", "medusa_accept_workspace_bytes",
    "medusa_accept", "medusa_accept_sampled", "medusa_verify_stats_bytes", "medusa_verify_fused_available",
    "medusa_verify_logits", "medusa_accept_fused", "kv_commit", "medusa_carry_over", "tree_linear_workspace_bytes", "tree_linear", "tree_linear_segments", "tree_linear_swiglu", "tree_interleave_gate_up", "tree_rope",
    "medusa_heads_timed",
    "medusa_gemm_plan",
)


class MedusaError(RuntimeError):
    pass


def library_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib_handle
    if _lib_handle is None:
        if not os.path.exists(_LIB_PATH):
            raise MedusaError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2401_10774_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        L = ctypes.CDLL(_LIB_PATH)
        c_int, c_void_p, c_size_t, c_float = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
        L.medusa_status_string.restype = ctypes.c_char_p
        L.medusa_status_string.argtypes = [c_int]
        L.medusa_tree_create_cartesian.argtypes = [c_void_p, c_int, ctypes.POINTER(c_void_p)]
        L.medusa_tree_create_nodes.argtypes = [c_void_p, c_int, c_int, ctypes.POINTER(c_void_p)]
        L.medusa_tree_create_optimized.argtypes = [c_void_p, c_int, c_int, c_int, ctypes.POINTER(c_void_p), c_void_p]
        L.medusa_tree_destroy.argtypes = [c_void_p]
        L.medusa_tree_query.argtypes = [c_void_p] + [c_void_p] * 5
        L.medusa_tree_tables.argtypes = [c_void_p] + [c_void_p] * 6
        L.medusa_heads.argtypes = [c_void_p] * 5 + [c_int] * 5 + [c_void_p]
        L.medusa_topk_tree_workspace_bytes.restype = c_size_t
        L.medusa_topk_tree_workspace_bytes.argtypes = [c_int, c_int]
        L.medusa_topk_tree.argtypes = [c_void_p] * 4 + [c_int] * 3 + [c_void_p] * 4 + [c_size_t, c_void_p]
        L.tree_attention_workspace_bytes.restype = c_size_t
        L.tree_attention_workspace_bytes.argtypes = [c_int] * 6
        L.tree_attention.argtypes = [c_void_p] * 8 + [c_int] * 5 + [c_float, c_int, c_void_p, c_size_t, c_void_p]
        L.tree_attention_static.argtypes = [c_void_p] * 8 + [c_int] * 5 + [c_float, c_int, c_void_p]
        L.tree_attention_static_scratch_bytes.restype = c_size_t
        L.tree_attention_static_scratch_bytes.argtypes = []
        L.medusa_accept_workspace_bytes.restype = c_size_t
        L.medusa_accept_workspace_bytes.argtypes = [c_int] * 3
        L.medusa_accept.argtypes = ([c_void_p] * 3 + [c_int] * 3 + [c_float] * 3 + [c_void_p] * 5 +
                                    [c_void_p, c_size_t, c_void_p])
        L.medusa_verify_stats_bytes.restype = c_size_t
        L.medusa_verify_stats_bytes.argtypes = [c_int, c_int]
        L.medusa_verify_fused_available.argtypes = [c_int] * 4
        L.medusa_verify_logits.argtypes = [c_void_p] * 4 + [c_size_t] + [c_int] * 5 + [c_float, c_void_p]
        L.medusa_accept_fused.argtypes = [c_void_p] * 4 + [c_int] * 3 + [c_float] * 3 + [c_void_p] * 5 + [c_void_p]
        L.medusa_accept_sampled.argtypes = ([c_void_p] * 4 + [c_int] * 2 + [c_float] + [c_void_p] * 5 +
                                            [c_void_p, c_size_t, c_void_p])
        L.kv_commit.argtypes = ([c_void_p] * 5 + [c_int, c_void_p, c_void_p, c_void_p] + [c_int] * 6 + [c_int, c_void_p])
        L.medusa_carry_over.argtypes = [c_void_p] * 5 + [c_int] * 5 + [c_void_p]
        L.tree_linear_workspace_bytes.restype = c_size_t
        L.tree_linear_workspace_bytes.argtypes = [c_int] * 5
        L.tree_linear.argtypes = [c_void_p] * 4 + [c_int] * 7 + [c_void_p, c_size_t, c_void_p]
        L.tree_linear_swiglu.argtypes = [c_void_p] * 3 + [c_int] * 7 + [c_void_p]
        L.tree_interleave_gate_up.argtypes = [c_void_p] * 3 + [c_int] * 3 + [c_void_p]
        L.tree_linear_segments.argtypes = [c_void_p] * 4 + [c_int] * 7 + [c_size_t, c_int, c_void_p, c_size_t, c_void_p]
        L.tree_rope.argtypes = [c_void_p] * 3 + [c_int] * 5 + [c_float, c_int, c_void_p]
        L.medusa_heads_timed.argtypes = [c_void_p] * 5 + [c_int] * 5 + [c_void_p] * 4
        L.medusa_gemm_plan.argtypes = [c_int] * 5 + [ctypes.POINTER(c_int)]
        for name in EXPORTED_SYMBOLS:
            fn = getattr(L, name)
            if fn.restype is ctypes.c_int or fn.restype is None:
                fn.restype = c_int
        _lib_handle = L
    return _lib_handle


def _check(status: int, what: str) -> None:
    if status != 0:
        msg = lib().medusa_status_string(status).decode()
        raise MedusaError(f"{what} failed: {msg} ({status})")


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MEDUSA_F32
    if t.dtype == torch.bfloat16:
        return MEDUSA_BF16
    raise MedusaError(f"unsupported storage dtype {t.dtype}")


def _dev(t: Optional[torch.Tensor], name: str, dtype=None, shape: Optional[Sequence[int]] = None) -> Optional[int]:
    """Pointer of a device tensor after checking residency, density, dtype and shape."""
    if t is None:
        return None
    if not t.is_cuda:
        raise MedusaError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise MedusaError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise MedusaError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise MedusaError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def _scratch(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


class MedusaTree:
    """Handle of a candidate tree (Sec. 2.1.2) plus host copies of its tables."""

    def __init__(self, branching: Optional[Sequence[int]] = None, nodes: Optional[Sequence[Sequence[int]]] = None,
                 accuracy=None, n_nodes: Optional[int] = None):
        L = lib()
        handle = ctypes.c_void_p()
        self.expected_accept_len = None
        if sum(x is not None for x in (branching, nodes, accuracy)) != 1:
            raise MedusaError("give exactly one of branching / nodes / accuracy")
        if accuracy is not None:
            acc = np.ascontiguousarray(accuracy, dtype=np.float64)
            if acc.ndim != 2 or n_nodes is None:
                raise MedusaError("accuracy must be a [K][S] table and n_nodes given")
            expect = ctypes.c_double()
            _check(L.medusa_tree_create_optimized(acc.ctypes.data, acc.shape[0], acc.shape[1], int(n_nodes),
                                                  ctypes.byref(handle), ctypes.addressof(expect)),
                   "medusa_tree_create_optimized")
            self.expected_accept_len = expect.value
        elif branching is not None:
            arr = np.ascontiguousarray(branching, dtype=np.int32)
            _check(L.medusa_tree_create_cartesian(arr.ctypes.data, int(arr.size), ctypes.byref(handle)),
                   "medusa_tree_create_cartesian")
        else:
            K = max((len(n) for n in nodes), default=0)
            arr = np.full((len(nodes), max(K, 1)), -1, np.int32)
            for i, n in enumerate(nodes):
                arr[i, :len(n)] = n
            _check(L.medusa_tree_create_nodes(arr.ctypes.data, len(nodes), K, ctypes.byref(handle)),
                   "medusa_tree_create_nodes")
        self._h = handle
        T, K, nl, S = (ctypes.c_int32() for _ in range(4))
        topk = np.zeros(8, np.int32)
        _check(L.medusa_tree_query(self._h, ctypes.addressof(T), ctypes.addressof(K), ctypes.addressof(nl),
                                   ctypes.addressof(S), topk.ctypes.data), "medusa_tree_query")
        self.T, self.K, self.n_leaves, self.S = T.value, K.value, nl.value, S.value
        self.topk_per_head = topk[:self.K].copy()
        self.parent = np.zeros(self.T, np.int32)
        self.depth = np.zeros(self.T, np.int32)
        self.rank = np.zeros(self.T, np.int32)
        self.token_src = np.zeros(self.T, np.int32)
        self.anc_mask = np.zeros((self.T, 2), np.uint64)
        self.paths = np.zeros((self.n_leaves, self.K + 1), np.int32)
        _check(L.medusa_tree_tables(self._h, self.parent.ctypes.data, self.depth.ctypes.data, self.rank.ctypes.data,
                                    self.token_src.ctypes.data, self.anc_mask.ctypes.data, self.paths.ctypes.data),
               "medusa_tree_tables")

    @property
    def handle(self):
        return self._h

    def close(self):
        if getattr(self, "_h", None):
            lib().medusa_tree_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def medusa_heads(hidden: torch.Tensor, w1: Optional[torch.Tensor], w2: torch.Tensor,
                 resid: Optional[torch.Tensor] = None, logits: Optional[torch.Tensor] = None, stream=None):
    """logits[m,k,:] = W2_k (SiLU(W1_k h_m) + h_m); w1=None gives W2_k h_m.  Returns (logits, resid)."""
    M, d = hidden.shape
    K, V, _ = w2.shape
    code = _dtype_code(hidden)
    _dev(hidden, "hidden", shape=(M, d))
    _dev(w2, "w2", dtype=hidden.dtype, shape=(K, V, d))
    if w1 is not None:
        _dev(w1, "w1", dtype=hidden.dtype, shape=(K, d, d))
        if resid is None:
            resid = torch.empty((M, K, d), dtype=hidden.dtype, device=hidden.device)
        _dev(resid, "resid", dtype=hidden.dtype, shape=(M, K, d))
    if logits is None:
        logits = torch.empty((M, K, V), dtype=torch.float32, device=hidden.device)
    _dev(logits, "logits", dtype=torch.float32, shape=(M, K, V))
    _check(lib().medusa_heads(hidden.data_ptr(), None if w1 is None else w1.data_ptr(), w2.data_ptr(),
                              None if w1 is None else resid.data_ptr(), logits.data_ptr(), M, d, V, K, code,
                              _stream(stream)), "medusa_heads")
    return logits, resid


def medusa_topk_tree(medusa_logits: torch.Tensor, lm_logits: torch.Tensor, tree: MedusaTree, prefix_len: torch.Tensor,
                     topk_ids=None, tree_tokens=None, position_ids=None, workspace=None, stream=None):
    """Returns (topk_ids [B,K,S], tree_tokens [B,T], position_ids [B,T]), all int32."""
    B, V = lm_logits.shape
    K_heads = medusa_logits.shape[1]
    dev = lm_logits.device
    _dev(medusa_logits, "medusa_logits", dtype=torch.float32, shape=(B, K_heads, V))
    _dev(lm_logits, "lm_logits", dtype=torch.float32)
    _dev(prefix_len, "prefix_len", dtype=torch.int32, shape=(B,))
    if topk_ids is None:
        topk_ids = torch.empty((B, tree.K, max(tree.S, 1)), dtype=torch.int32, device=dev)
    if tree_tokens is None:
        tree_tokens = torch.empty((B, tree.T), dtype=torch.int32, device=dev)
    if position_ids is None:
        position_ids = torch.empty((B, tree.T), dtype=torch.int32, device=dev)
    _dev(topk_ids, "topk_ids", dtype=torch.int32)
    _dev(tree_tokens, "tree_tokens", dtype=torch.int32, shape=(B, tree.T))
    _dev(position_ids, "position_ids", dtype=torch.int32, shape=(B, tree.T))
    if workspace is None:
        workspace = _scratch(lib().medusa_topk_tree_workspace_bytes(B, tree.K), dev)
    _dev(workspace, "workspace")
    _check(lib().medusa_topk_tree(medusa_logits.data_ptr(), lm_logits.data_ptr(), tree.handle, prefix_len.data_ptr(),
                                  B, V, K_heads, topk_ids.data_ptr(), tree_tokens.data_ptr(), position_ids.data_ptr(),
                                  workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream)),
           "medusa_topk_tree")
    return topk_ids, tree_tokens, position_ids


def tree_attention_workspace_bytes(B: int, Hq: int, Hkv: int, T: int, D: int, Lcap: int) -> int:
    return int(lib().tree_attention_workspace_bytes(B, Hq, Hkv, T, D, Lcap))


def tree_attention(q: torch.Tensor, k_tree: torch.Tensor, v_tree: torch.Tensor, k_cache: torch.Tensor,
                   v_cache: torch.Tensor, prefix_len: torch.Tensor, tree: MedusaTree, scale: float,
                   out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """Tree-masked attention of the T tree tokens over one layer's cache.  Returns out [B,Hq,T,D]."""
    B, Hq, T, D = q.shape
    Hkv, Lcap = k_cache.shape[1], k_cache.shape[2]
    if T != tree.T:
        raise MedusaError(f"q has {T} tree tokens, the tree has {tree.T}")
    code = _dtype_code(q)
    _dev(q, "q")
    _dev(k_tree, "k_tree", dtype=q.dtype, shape=(B, Hkv, T, D))
    _dev(v_tree, "v_tree", dtype=q.dtype, shape=(B, Hkv, T, D))
    _dev(k_cache, "k_cache", dtype=q.dtype, shape=(B, Hkv, Lcap, D))
    _dev(v_cache, "v_cache", dtype=q.dtype, shape=(B, Hkv, Lcap, D))
    _dev(prefix_len, "prefix_len", dtype=torch.int32, shape=(B,))
    if out is None:
        out = torch.empty_like(q)
    _dev(out, "out", dtype=q.dtype, shape=(B, Hq, T, D))
    if workspace is None:
        workspace = _scratch(tree_attention_workspace_bytes(B, Hq, Hkv, T, D, Lcap), q.device)
    _dev(workspace, "workspace")
    _check(lib().tree_attention(q.data_ptr(), k_tree.data_ptr(), v_tree.data_ptr(), k_cache.data_ptr(),
                                v_cache.data_ptr(), prefix_len.data_ptr(), tree.handle, out.data_ptr(), B, Hq, Hkv, D,
                                Lcap, float(scale), code, workspace.data_ptr(),
                                workspace.numel() * workspace.element_size(), _stream(stream)), "tree_attention")
    return out


def tree_attention_static(q: torch.Tensor, k_tree: torch.Tensor, v_tree: torch.Tensor, k_cache: torch.Tensor,
                          v_cache: torch.Tensor, prefix_len: torch.Tensor, tree: MedusaTree, scale: float,
                          out: torch.Tensor, stream=None) -> torch.Tensor:
    """tree_attention on the library's built-in scratch array: the call allocates nothing, so `out` is
    required.  Raises MedusaError (MEDUSA_ESCRATCH) for shapes whose split partials exceed the array."""
    B, Hq, T, D = q.shape
    Hkv, Lcap = k_cache.shape[1], k_cache.shape[2]
    if T != tree.T:
        raise MedusaError(f"q has {T} tree tokens, the tree has {tree.T}")
    code = _dtype_code(q)
    _dev(q, "q")
    _dev(k_tree, "k_tree", dtype=q.dtype, shape=(B, Hkv, T, D))
    _dev(v_tree, "v_tree", dtype=q.dtype, shape=(B, Hkv, T, D))
    _dev(k_cache, "k_cache", dtype=q.dtype, shape=(B, Hkv, Lcap, D))
    _dev(v_cache, "v_cache", dtype=q.dtype, shape=(B, Hkv, Lcap, D))
    _dev(prefix_len, "prefix_len", dtype=torch.int32, shape=(B,))
    _dev(out, "out", dtype=q.dtype, shape=(B, Hq, T, D))
    _check(lib().tree_attention_static(q.data_ptr(), k_tree.data_ptr(), v_tree.data_ptr(), k_cache.data_ptr(),
                                       v_cache.data_ptr(), prefix_len.data_ptr(), tree.handle, out.data_ptr(), B, Hq, Hkv,
                                       D, Lcap, float(scale), code, _stream(stream)), "tree_attention_static")
    return out


def medusa_accept_workspace_bytes(B: int, T: int, V: int) -> int:
    return int(lib().medusa_accept_workspace_bytes(B, T, V))


def medusa_accept(logits: torch.Tensor, tree_tokens: torch.Tensor, tree: MedusaTree, mode: str = "greedy",
                  temperature: float = 1.0, eps: float = 0.0, delta: float = 0.0, outputs=None, workspace=None,
                  stream=None):
    """Returns (accept_len [B], best_node [B], path_nodes [B,K+1], accepted_tokens [B,K+1], next_root [B])."""
    B, T, V = logits.shape
    if T != tree.T:
        raise MedusaError(f"logits have {T} rows per sequence, the tree has {tree.T}")
    dev = logits.device
    _dev(logits, "logits", dtype=torch.float32)
    _dev(tree_tokens, "tree_tokens", dtype=torch.int32, shape=(B, T))
    if outputs is None:
        i32 = dict(dtype=torch.int32, device=dev)
        outputs = (torch.empty(B, **i32), torch.empty(B, **i32), torch.empty((B, tree.K + 1), **i32),
                   torch.empty((B, tree.K + 1), **i32), torch.empty(B, **i32))
    accept_len, best_node, path_nodes, accepted_tokens, next_root = outputs
    _dev(accept_len, "accept_len", dtype=torch.int32, shape=(B,))
    _dev(best_node, "best_node", dtype=torch.int32, shape=(B,))
    _dev(path_nodes, "path_nodes", dtype=torch.int32, shape=(B, tree.K + 1))
    _dev(accepted_tokens, "accepted_tokens", dtype=torch.int32, shape=(B, tree.K + 1))
    _dev(next_root, "next_root", dtype=torch.int32, shape=(B,))
    if workspace is None:
        workspace = _scratch(medusa_accept_workspace_bytes(B, T, V), dev)
    _dev(workspace, "workspace")
    code = {"greedy": MEDUSA_GREEDY, "typical": MEDUSA_TYPICAL}[mode]
    _check(lib().medusa_accept(logits.data_ptr(), tree_tokens.data_ptr(), tree.handle, B, V, code, float(temperature),
                               float(eps), float(delta), accept_len.data_ptr(), best_node.data_ptr(),
                               path_nodes.data_ptr(), accepted_tokens.data_ptr(), next_root.data_ptr(),
                               workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream)),
           "medusa_accept")
    return outputs


def medusa_verify_fused_available(M: int, d: int, V: int, dtype: torch.dtype) -> bool:
    return bool(lib().medusa_verify_fused_available(M, d, V, 1 if dtype == torch.bfloat16 else 0))


def medusa_verify_logits(hidden_tree: torch.Tensor, w_lm: torch.Tensor, mode: str = "greedy", temperature: float = 1.0,
                         logits: Optional[torch.Tensor] = None, stats: Optional[torch.Tensor] = None, stream=None):
    """LM-head logits of the tree rows [M, d] x [V, d] plus the acceptance step's row reductions.  Returns (logits [M, V], stats)."""
    M, d = hidden_tree.shape
    V = w_lm.shape[0]
    _dev(hidden_tree, "hidden_tree")
    _dev(w_lm, "w_lm", dtype=hidden_tree.dtype, shape=(V, d))
    if logits is None:
        logits = torch.empty((M, V), dtype=torch.float32, device=hidden_tree.device)
    _dev(logits, "logits", dtype=torch.float32)
    if stats is None:
        stats = _scratch(lib().medusa_verify_stats_bytes(M, V), hidden_tree.device)
    _dev(stats, "stats")
    code = {"greedy": MEDUSA_GREEDY, "typical": MEDUSA_TYPICAL}[mode]
    _check(lib().medusa_verify_logits(hidden_tree.data_ptr(), w_lm.data_ptr(), logits.data_ptr(), stats.data_ptr(),
                                      stats.numel() * stats.element_size(), M, d, V, _dtype_code(hidden_tree), code,
                                      float(temperature), _stream(stream)), "medusa_verify_logits")
    return logits, stats


def medusa_accept_fused(logits: torch.Tensor, stats: torch.Tensor, tree_tokens: torch.Tensor, tree: MedusaTree,
                        mode: str = "greedy", temperature: float = 1.0, eps: float = 0.0, delta: float = 0.0, outputs=None,
                        stream=None):
    """medusa_accept from the row reductions medusa_verify_logits left in `stats`.  logits [B, T, V]."""
    B, T, V = logits.shape
    if T != tree.T:
        raise MedusaError(f"logits have {T} rows per sequence, the tree has {tree.T}")
    _dev(logits, "logits", dtype=torch.float32)
    _dev(stats, "stats")
    _dev(tree_tokens, "tree_tokens", dtype=torch.int32, shape=(B, T))
    if outputs is None:
        i32 = dict(dtype=torch.int32, device=logits.device)
        outputs = (torch.empty(B, **i32), torch.empty(B, **i32), torch.empty((B, tree.K + 1), **i32),
                   torch.empty((B, tree.K + 1), **i32), torch.empty(B, **i32))
    for o, name, shape in zip(outputs, ("accept_len", "best_node", "path_nodes", "accepted_tokens", "next_root"),
                              ((B,), (B,), (B, tree.K + 1), (B, tree.K + 1), (B,))):
        _dev(o, name, dtype=torch.int32, shape=shape)
    code = {"greedy": MEDUSA_GREEDY, "typical": MEDUSA_TYPICAL}[mode]
    _check(lib().medusa_accept_fused(logits.data_ptr(), stats.data_ptr(), tree_tokens.data_ptr(), tree.handle, B, V, code,
                                     float(temperature), float(eps), float(delta), *(o.data_ptr() for o in outputs),
                                     _stream(stream)), "medusa_accept_fused")
    return outputs


def medusa_accept_sampled(logits: torch.Tensor, tree_tokens: torch.Tensor, tree: MedusaTree, uniforms: torch.Tensor,
                          temperature: float = 1.0, outputs=None, workspace=None, stream=None):
    """Rejection-sampling acceptance with caller-supplied uniforms [B, T] (slot 0 of a row draws the next
    token).  Returns (accept_len [B], best_node [B], path_nodes [B,K+1], accepted_tokens [B,K+1], next_token [B])."""
    B, T, V = logits.shape
    if T != tree.T:
        raise MedusaError(f"logits have {T} rows per sequence, the tree has {tree.T}")
    dev = logits.device
    _dev(logits, "logits", dtype=torch.float32)
    _dev(tree_tokens, "tree_tokens", dtype=torch.int32, shape=(B, T))
    _dev(uniforms, "uniforms", dtype=torch.float32, shape=(B, T))
    if outputs is None:
        i32 = dict(dtype=torch.int32, device=dev)
        outputs = (torch.empty(B, **i32), torch.empty(B, **i32), torch.empty((B, tree.K + 1), **i32),
                   torch.empty((B, tree.K + 1), **i32), torch.empty(B, **i32))
    for o, name, shape in zip(outputs, ("accept_len", "best_node", "path_nodes", "accepted_tokens", "next_token"),
                              ((B,), (B,), (B, tree.K + 1), (B, tree.K + 1), (B,))):
        _dev(o, name, dtype=torch.int32, shape=shape)
    if workspace is None:
        workspace = _scratch(medusa_accept_workspace_bytes(B, T, V), dev)
    _dev(workspace, "workspace")
    _check(lib().medusa_accept_sampled(logits.data_ptr(), tree_tokens.data_ptr(), tree.handle, uniforms.data_ptr(), B, V,
                                       float(temperature), *(o.data_ptr() for o in outputs), workspace.data_ptr(),
                                       workspace.numel() * workspace.element_size(), _stream(stream)),
           "medusa_accept_sampled")
    return outputs


def kv_commit(k_cache: torch.Tensor, v_cache: torch.Tensor, k_tree: torch.Tensor, v_tree: torch.Tensor,
              path_nodes: torch.Tensor, accept_len: torch.Tensor, prefix_len: torch.Tensor,
              prefix_len_out: Optional[torch.Tensor] = None, stream=None) -> None:
    """Append the accepted path's K/V rows to every cache layer and advance prefix_len (in place, or
    into prefix_len_out)."""
    NL, B, Hkv, Lcap, D = k_cache.shape
    T = k_tree.shape[3]
    code = _dtype_code(k_cache)
    _dev(k_cache, "k_cache")
    _dev(v_cache, "v_cache", dtype=k_cache.dtype, shape=(NL, B, Hkv, Lcap, D))
    _dev(k_tree, "k_tree", dtype=k_cache.dtype, shape=(NL, B, Hkv, T, D))
    _dev(v_tree, "v_tree", dtype=k_cache.dtype, shape=(NL, B, Hkv, T, D))
    _dev(path_nodes, "path_nodes", dtype=torch.int32)
    if path_nodes.dim() != 2 or path_nodes.shape[0] != B:
        raise MedusaError("path_nodes must be [B, K+1]")
    _dev(accept_len, "accept_len", dtype=torch.int32, shape=(B,))
    _dev(prefix_len, "prefix_len", dtype=torch.int32, shape=(B,))
    if prefix_len_out is not None:
        _dev(prefix_len_out, "prefix_len_out", dtype=torch.int32, shape=(B,))
    _check(lib().kv_commit(k_cache.data_ptr(), v_cache.data_ptr(), k_tree.data_ptr(), v_tree.data_ptr(),
                           path_nodes.data_ptr(), int(path_nodes.shape[1]), accept_len.data_ptr(),
                           prefix_len.data_ptr(), None if prefix_len_out is None else prefix_len_out.data_ptr(),
                           NL, B, Hkv, T, D, Lcap, code, _stream(stream)), "kv_commit")


def medusa_carry_over(hidden_tree: Optional[torch.Tensor], verify_logits: Optional[torch.Tensor], best_node: torch.Tensor,
                      h_next: Optional[torch.Tensor] = None, lm_next: Optional[torch.Tensor] = None, stream=None):
    """The next step's starting activations: rows best_node[b] of hidden_tree [B,T,d] and of verify_logits
    [B,T,V] gathered into h_next [B,d] and lm_next [B,V] (allocated when missing).  Returns (h_next, lm_next)."""
    B = best_node.shape[0]
    _dev(best_node, "best_node", dtype=torch.int32, shape=(B,))
    T = d = V = 0
    code = MEDUSA_F32
    if hidden_tree is not None:
        _, T, d = hidden_tree.shape
        code = _dtype_code(hidden_tree)
        _dev(hidden_tree, "hidden_tree", shape=(B, T, d))
        if h_next is None:
            h_next = torch.empty((B, d), dtype=hidden_tree.dtype, device=hidden_tree.device)
        _dev(h_next, "h_next", dtype=hidden_tree.dtype, shape=(B, d))
    if verify_logits is not None:
        _, T, V = verify_logits.shape
        _dev(verify_logits, "verify_logits", dtype=torch.float32, shape=(B, T, V))
        if lm_next is None:
            lm_next = torch.empty((B, V), dtype=torch.float32, device=verify_logits.device)
        _dev(lm_next, "lm_next", dtype=torch.float32, shape=(B, V))
    _check(lib().medusa_carry_over(None if hidden_tree is None else hidden_tree.data_ptr(),
                                   None if verify_logits is None else verify_logits.data_ptr(), best_node.data_ptr(),
                                   None if hidden_tree is None else h_next.data_ptr(),
                                   None if verify_logits is None else lm_next.data_ptr(), B, T, d, V, code, _stream(stream)),
           "medusa_carry_over")
    return h_next, lm_next


def tree_linear_workspace_bytes(B: int, T: int, d_in: int, d_out: int, dtype: torch.dtype) -> int:
    code = 1 if dtype == torch.bfloat16 else 0
    return int(lib().tree_linear_workspace_bytes(B, T, d_in, d_out, code))


def tree_linear(x: torch.Tensor, w: torch.Tensor, B: int, T: int, mul: Optional[torch.Tensor] = None,
                y: Optional[torch.Tensor] = None, y_heads: int = 0, workspace: Optional[torch.Tensor] = None,
                stream=None) -> torch.Tensor:
    """y = x w^T (or SiLU(x w^T) * mul) on the B*T tree tokens.  x is token-major [B*T, d_in] or
    head-major [B, H, T, Dh] (as tree_attention writes it); y is token-major [B*T, d_out] or, with
    y_heads > 0, head-major [B, y_heads, T, d_out / y_heads]."""
    code = _dtype_code(x)
    d_out, d_in = w.shape
    if x.dim() == 2:
        x_heads = 0
        _dev(x, "x", shape=(B * T, d_in))
    elif x.dim() == 4:
        x_heads = int(x.shape[1])
        _dev(x, "x", shape=(B, x_heads, T, d_in // max(x_heads, 1)))
    else:
        raise MedusaError("x must be [B*T, d_in] or [B, H, T, Dh]")
    _dev(w, "w", dtype=x.dtype, shape=(d_out, d_in))
    if mul is not None:
        _dev(mul, "mul", dtype=x.dtype, shape=(B * T, d_out))
    shape = (B * T, d_out) if y_heads == 0 else (B, y_heads, T, d_out // y_heads)
    if y is None:
        y = torch.empty(shape, dtype=x.dtype, device=x.device)
    _dev(y, "y", dtype=x.dtype, shape=shape)
    if workspace is None:
        need = tree_linear_workspace_bytes(B, T, d_in, d_out, x.dtype)
        workspace = _scratch(need, x.device) if need else None
    _check(lib().tree_linear(x.data_ptr(), w.data_ptr(), None if mul is None else mul.data_ptr(), y.data_ptr(),
                             B, T, d_in, d_out, x_heads, y_heads, code,
                             None if workspace is None else workspace.data_ptr(),
                             0 if workspace is None else workspace.numel() * workspace.element_size(),
                             _stream(stream)), "tree_linear")
    return y


def tree_linear_segments(x: torch.Tensor, w: torch.Tensor, B: int, T: int, y: torch.Tensor, y_heads: int,
                         workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """One projection call for several head-major outputs (Q, K, V): w is the stacked weight
    [segments * y_heads * Dh, d_in] and y one tensor [segments, B, y_heads, T, Dh] whose slices y[s]
    are the outputs.  x as for tree_linear."""
    code = _dtype_code(x)
    d_out, d_in = w.shape
    if x.dim() == 2:
        x_heads = 0
        _dev(x, "x", shape=(B * T, d_in))
    elif x.dim() == 4:
        x_heads = int(x.shape[1])
        _dev(x, "x", shape=(B, x_heads, T, d_in // max(x_heads, 1)))
    else:
        raise MedusaError("x must be [B*T, d_in] or [B, H, T, Dh]")
    _dev(w, "w", dtype=x.dtype, shape=(d_out, d_in))
    if y.dim() != 5 or y_heads < 1 or d_out % (int(y.shape[0]) * y_heads) != 0:
        raise MedusaError("y must be [segments, B, y_heads, T, Dh] with segments * y_heads * Dh == d_out")
    segments = int(y.shape[0])
    _dev(y, "y", dtype=x.dtype, shape=(segments, B, y_heads, T, d_out // (segments * y_heads)))
    if workspace is None:
        need = tree_linear_workspace_bytes(B, T, d_in, d_out, x.dtype)
        workspace = _scratch(need, x.device) if need else None
    _check(lib().tree_linear_segments(x.data_ptr(), w.data_ptr(), None, y.data_ptr(), B, T, d_in, d_out, x_heads, y_heads,
                                      segments, y[0].numel(), code,
                                      None if workspace is None else workspace.data_ptr(),
                                      0 if workspace is None else workspace.numel() * workspace.element_size(),
                                      _stream(stream)), "tree_linear_segments")
    return y


def interleave_gate_up(w_gate: torch.Tensor, w_up: torch.Tensor, stream=None) -> torch.Tensor:
    """The weight layout tree_linear_swiglu reads: blocks of 16 gate rows followed by the same 16 rows
    of the up projection.  [d_out, d_in] x 2 -> [2*d_out, d_in]; d_out a multiple of 16."""
    d_out, d_in = w_gate.shape
    if w_up.shape != w_gate.shape or d_out % 16 != 0:
        raise MedusaError("gate and up weights must have the same shape, rows a multiple of 16")
    _dev(w_gate, "w_gate", shape=(d_out, d_in))
    _dev(w_up, "w_up", dtype=w_gate.dtype, shape=(d_out, d_in))
    w_gu = torch.empty((2 * d_out, d_in), dtype=w_gate.dtype, device=w_gate.device)
    _check(lib().tree_interleave_gate_up(w_gate.data_ptr(), w_up.data_ptr(), w_gu.data_ptr(), d_out, d_in, _dtype_code(w_gate),
                                         _stream(stream)), "tree_interleave_gate_up")
    return w_gu


def tree_linear_swiglu(x: torch.Tensor, w_gu: torch.Tensor, B: int, T: int, y: Optional[torch.Tensor] = None,
                       y_heads: int = 0, stream=None) -> torch.Tensor:
    """y = SiLU(x w_g^T) * (x w_u^T) in one pass; w_gu = interleave_gate_up(w_g, w_u).  x token-major
    [B*T, d_in] or head-major [B, H, T, Dh]; y token-major [B*T, d_out] or head-major."""
    code = _dtype_code(x)
    d_out, d_in = w_gu.shape[0] // 2, w_gu.shape[1]
    _dev(w_gu, "w_gu", dtype=x.dtype, shape=(2 * d_out, d_in))
    x_heads = 0
    if x.dim() == 4:
        if x.shape[0] != B or x.shape[2] != T or x.shape[1] * x.shape[3] != d_in:
            raise MedusaError("head-major x must be [B, H, T, d_in/H]")
        x_heads = int(x.shape[1])
        _dev(x, "x", dtype=x.dtype)
    else:
        _dev(x, "x", dtype=x.dtype, shape=(B * T, d_in))
    if y is None:
        y = torch.empty((B, y_heads, T, d_out // y_heads) if y_heads > 0 else (B * T, d_out), dtype=x.dtype, device=x.device)
    _dev(y, "y", dtype=x.dtype)
    if y.numel() != B * T * d_out:
        raise MedusaError("y has the wrong number of elements")
    _check(lib().tree_linear_swiglu(x.data_ptr(), w_gu.data_ptr(), y.data_ptr(), B, T, d_in, d_out, x_heads, y_heads, code,
                                    _stream(stream)), "tree_linear_swiglu")
    return y


def medusa_gemm_plan(M: int, N: int, d: int, K: int = 1, have_workspace: bool = True) -> dict:
    """Which kernel arrangement a bf16 product of M rows with K matrices of N x d would get
    (host-side diagnostic, no GPU work)."""
    out = (ctypes.c_int * 6)()
    _check(lib().medusa_gemm_plan(int(M), int(N), int(d), int(K), int(bool(have_workspace)), out), "medusa_gemm_plan")
    kinds = ("gemv", "skinny", "square", "big")
    return {"kind": kinds[out[0]], "tile": out[1], "wide": (out[0] == 1 and out[1] == 128) or (out[0] == 3 and out[1] == 192), "ring": bool(out[2]), "mt": out[3],
            "m_blocks": out[4], "ksplit": out[5]}


def tree_rope(q: torch.Tensor, k: torch.Tensor, position_ids: torch.Tensor, theta: float = 10000.0, stream=None) -> None:
    """Rotary embedding of q [B, Hq, T, D] and k [B, Hkv, T, D] in place at position_ids [B, T] (int32)."""
    B, Hq, T, D = q.shape
    Hkv = k.shape[1]
    code = _dtype_code(q)
    _dev(q, "q")
    _dev(k, "k", dtype=q.dtype, shape=(B, Hkv, T, D))
    _dev(position_ids, "position_ids", dtype=torch.int32, shape=(B, T))
    _check(lib().tree_rope(q.data_ptr(), k.data_ptr(), position_ids.data_ptr(), B, Hq, Hkv, T, D, float(theta), code,
                           _stream(stream)), "tree_rope")
