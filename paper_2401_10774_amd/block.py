"""The simplified decoder block of App. G on the tree tokens, chained from the library's calls:
X W_Q, X W_K, X W_V (tree_linear), rotary embedding at the tree positions (tree_rope), Q K^T and
P V against the cache (tree_attention), X W_u, X W_g, X W_d (tree_linear).  Buffers are allocated
once and the calls' arguments are marshalled once per set of operands; ``run`` only launches
kernels.  Argument marshalling only -- every operator runs in the HIP library.

With one sequence, and W_Q, W_K, W_V handed in as consecutive row blocks of one allocation (views
of a [(Hq + 2 Hkv) D, h] tensor), the three projections are one tree_linear call: its head-major
output [1, Hq + 2 Hkv, T, D] is q, k and v back to back.  With ``w_gu`` (binding.interleave_gate_up
of W_g and W_u) given and at most 192 tree tokens in all (or a batch that the large-tile kernel takes), X W_u and X W_g are one
tree_linear_swiglu call and ``self.up`` is not produced."""
from __future__ import annotations

import torch

from . import binding as _b


class SimplifiedBlock:
    def __init__(self, tree: "_b.MedusaTree", B: int, h: int, Hq: int, Hkv: int, D: int, inter: int, Lcap: int,
                 dtype: torch.dtype, device="cuda", theta: float = 10000.0):
        self.tree, self.B, self.T = tree, B, tree.T
        self.h, self.Hq, self.Hkv, self.D, self.inter, self.Lcap, self.theta = h, Hq, Hkv, D, inter, Lcap, theta
        T = tree.T
        mk = lambda *shape: torch.empty(shape, dtype=dtype, device=device)
        if B == 1:
            self.qkv = mk(1, Hq + 2 * Hkv, T, D)
            self.q, self.k, self.v = self.qkv[:, :Hq], self.qkv[:, Hq:Hq + Hkv], self.qkv[:, Hq + Hkv:]
        elif Hq == Hkv:                        # three head-major tensors of one allocation: one projection call can fill them
            self.qkv = None
            self.qkv3 = mk(3, B, Hq, T, D)
            self.q, self.k, self.v = self.qkv3[0], self.qkv3[1], self.qkv3[2]
        else:                                  # grouped-query attention: K and V are the same size, Q is not
            self.qkv = None
            self.kv2 = mk(2, B, Hkv, T, D)
            self.q, self.k, self.v = mk(B, Hq, T, D), self.kv2[0], self.kv2[1]
        self.attn = mk(B, Hq, T, D)
        self.up, self.act, self.out = mk(B * T, inter), mk(B * T, inter), mk(B * T, h)
        self.ws = _b._scratch(_b.tree_attention_workspace_bytes(B, Hq, Hkv, T, D, Lcap), device)
        need = max(_b.tree_linear_workspace_bytes(B, T, d_in, d_out, dtype)
                   for d_in, d_out in ((h, Hq * D), (h, Hkv * D), (h, 2 * Hkv * D), (h, (Hq + 2 * Hkv) * D), (Hq * D, inter),
                                       (inter, h)))
        self.ws_lin = _b._scratch(need, device)
        self._plans = {}

    def _calls(self, x, wq, wk, wv, wu, wg, wd, k_cache, v_cache, prefix_len, position_ids, scale, w_gu=None, qkv=None, out=None):
        key = tuple(None if t is None else t.data_ptr() for t in (x, wq, wk, wv, wu, wg, wd, k_cache, v_cache, prefix_len, position_ids)) + (
            scale, None if w_gu is None else w_gu.data_ptr(), None if qkv is None else tuple(t.data_ptr() for t in qkv),
            None if out is None else out.data_ptr())
        plan = self._plans.get(key)
        if plan is not None:
            return plan
        dt = self.q.dtype
        B, T, h, Hq, Hkv, D, inter = self.B, self.T, self.h, self.Hq, self.Hkv, self.D, self.inter
        q_buf, k_buf, v_buf = (self.q, self.k, self.v) if qkv is None else qkv
        out_buf = self.out if out is None else out
        if qkv is not None:
            _b._dev(q_buf, "q", dtype=dt, shape=(B, Hq, T, D))
            _b._dev(k_buf, "k", dtype=dt, shape=(B, Hkv, T, D))
            _b._dev(v_buf, "v", dtype=dt, shape=(B, Hkv, T, D))
        if out is not None:
            _b._dev(out_buf, "out", dtype=dt, shape=(B * T, h))
        _b._dev(x, "x", dtype=dt, shape=(B * T, h))
        for name, w, shape in (("wq", wq, (Hq * D, h)), ("wk", wk, (Hkv * D, h)), ("wv", wv, (Hkv * D, h)),
                               ("wu", wu, (inter, Hq * D)), ("wg", wg, (inter, Hq * D)), ("wd", wd, (h, inter))):
            if w is not None or name not in ("wu", "wg"):        # (w_u and w_g may be left out when w_gu serves)
                _b._dev(w, name, dtype=dt, shape=shape)
        _b._dev(k_cache, "k_cache", dtype=dt, shape=(B, Hkv, self.Lcap, D))
        _b._dev(v_cache, "v_cache", dtype=dt, shape=(B, Hkv, self.Lcap, D))
        _b._dev(prefix_len, "prefix_len", dtype=torch.int32, shape=(B,))
        _b._dev(position_ids, "position_ids", dtype=torch.int32, shape=(B, T))
        L, code, p = _b.lib(), _b._dtype_code(x), (lambda t: t.data_ptr())
        nb = lambda t: t.numel() * t.element_size()
        lin = lambda xin, w, mul, y, d_in, d_out, xh, yh: (
            "tree_linear", L.tree_linear, (p(xin), p(w), None if mul is None else p(mul), p(y), B, T, d_in, d_out, xh, yh,
                                           code, p(self.ws_lin), nb(self.ws_lin)))
        nbytes = lambda t: t.numel() * t.element_size()
        # several head-major outputs of one projection call: segment s lands `stride` elements after segment s - 1
        seg = lambda w, y, stride, d_out, yh, n_seg: (
            "tree_linear_segments", L.tree_linear_segments, (p(x), p(w), None, p(y), B, T, h, d_out, 0, yh, n_seg, stride,
                                                             code, p(self.ws_lin), nb(self.ws_lin)))
        kv_adjacent = wv.data_ptr() == wk.data_ptr() + nbytes(wk)
        qkv_adjacent = kv_adjacent and wk.data_ptr() == wq.data_ptr() + nbytes(wq)
        es = q_buf.element_size()
        kv_stride = (v_buf.data_ptr() - k_buf.data_ptr()) // es      # caller-owned q, k, v: equally spaced tensors can share a call
        qk_stride = (k_buf.data_ptr() - q_buf.data_ptr()) // es
        if qkv is None and self.qkv is not None and qkv_adjacent:      # one sequence: q, k, v are head ranges of one head-major tensor
            qkv_calls = [lin(x, wq, None, self.qkv, h, (Hq + 2 * Hkv) * D, 0, Hq + 2 * Hkv)]
        elif qkv is None and B > 1 and Hq == Hkv and qkv_adjacent:     # a batch: three tensors, one call over the stacked weight rows
            qkv_calls = [seg(wq, self.qkv3, self.qkv3[0].numel(), 3 * Hq * D, Hq, 3)]
        elif qkv is None and B > 1 and Hq != Hkv and kv_adjacent:
            qkv_calls = [lin(x, wq, None, self.q, h, Hq * D, 0, Hq), seg(wk, self.kv2, self.kv2[0].numel(), 2 * Hkv * D, Hkv, 2)]
        elif qkv is not None and Hq == Hkv and qkv_adjacent and qk_stride == kv_stride and kv_stride >= k_buf.numel():
            qkv_calls = [seg(wq, q_buf, kv_stride, 3 * Hq * D, Hq, 3)]
        elif qkv is not None and kv_adjacent and kv_stride >= k_buf.numel():
            qkv_calls = [lin(x, wq, None, q_buf, h, Hq * D, 0, Hq), seg(wk, k_buf, kv_stride, 2 * Hkv * D, Hkv, 2)]
        else:
            qkv_calls = [lin(x, wq, None, q_buf, h, Hq * D, 0, Hq), lin(x, wk, None, k_buf, h, Hkv * D, 0, Hkv),
                         lin(x, wv, None, v_buf, h, Hkv * D, 0, Hkv)]
        plan = qkv_calls + [
            ("tree_rope", L.tree_rope, (p(q_buf), p(k_buf), p(position_ids), B, Hq, Hkv, T, D, float(self.theta), code)),
            ("tree_attention", L.tree_attention, (p(q_buf), p(k_buf), p(v_buf), p(k_cache), p(v_cache), p(prefix_len),
                                                  self.tree.handle, p(self.attn), B, Hq, Hkv, D, self.Lcap, float(scale),
                                                  code, p(self.ws), nb(self.ws))),
        ]
        # gate and up in one pass: up to 192 rows (one or two row blocks of the ring kernel) and wherever the
        # planning gives the stacked projection the large-tile kernel (measured at 7B and 13B shapes, 65 to 260 rows:
        # one pass always beats two calls, 45 against 61 us at 89 rows, 77 against 109 at 176); more row blocks of
        # the ring kernel than two are not measured: two calls then
        fuse_gu = w_gu is not None and (B * T <= 192 or _b.medusa_gemm_plan(B * T, 2 * inter, Hq * D, 1, False)["kind"] == "big")
        if fuse_gu:
            _b._dev(w_gu, "w_gu", dtype=dt, shape=(2 * inter, Hq * D))
            plan.append(("tree_linear_swiglu", L.tree_linear_swiglu, (p(self.attn), p(w_gu), p(self.act), B, T, Hq * D, inter,
                                                                      Hq, 0, code)))
        else:
            if wu is None or wg is None:
                raise _b.MedusaError("this row count takes two projection calls: w_u and w_g are needed")
            plan += [lin(self.attn, wu, None, self.up, Hq * D, inter, Hq, 0),
                     lin(self.attn, wg, self.up, self.act, Hq * D, inter, Hq, 0)]
        plan.append(lin(self.act, wd, None, out_buf, inter, h, 0, 0))
        self._plans[key] = plan
        return plan

    def run(self, x, wq, wk, wv, wu, wg, wd, k_cache, v_cache, prefix_len, position_ids, scale: float, w_gu=None,
            qkv=None, out=None):
        """x [B*T, h]; weights out x in; k_cache, v_cache [B, Hkv, Lcap, D] of one layer.  Enqueues the
        block on the current stream and returns its output [B*T, h]; intermediates stay in
        self.q/k/v/attn/up/act.  ``qkv`` = (q, k, v), caller-owned head-major tensors [B, H, T, D] the
        projections write instead of the block's own (a stack of layers keeps every layer's K and V of
        the tree tokens for kv_commit; equally spaced tensors over adjacent weights share one call);
        ``out`` = a caller-owned output [B*T, h] (not x)."""
        stream = torch.cuda.current_stream().cuda_stream
        for name, fn, args in self._calls(x, wq, wk, wv, wu, wg, wd, k_cache, v_cache, prefix_len, position_ids, scale, w_gu,
                                          qkv, out):
            rc = fn(*args, stream)
            if rc != 0:
                _b._check(rc, name)
        return self.out if out is None else out
