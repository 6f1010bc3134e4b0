"""Convenience holder for one Jigsaw linear layer's device buffers.

PyTorch is used for device memory and the stream only; every computation (shard,
forward, gather) is a call into ``libjigsaw`` through :mod:`binding`.
"""
from __future__ import annotations

import torch

from . import binding as jg


class JigsawLinear:
    """Plan + per-rank shard tensors (X_r, W_r, b_r, Y_r) + workspace on one GPU.

    ``op = JG_OP_XWT``: Y = X W^T with X (M, K) and W (N, K).  ``op = JG_OP_XW``: Y = X W with W (K, N).
    ``op = JG_OP_XTW``: the transposed
    layer Y = X^T W with X (K, M) and W (K, N).  ``dtype = JG_BF16 / JG_BF16X3``: the X and W shards are
    bfloat16 tensors (split mode: every row is [hi | lo]) written by ``shard`` from FP32 inputs; the backward of such a
    plan reads FP32 copies (``shard_master``).
    """

    def __init__(self, M: int, K: int, N: int, ways: int, bias: bool = False,
                 combine: int = jg.JG_COMBINE_FUSED, weights: int = jg.JG_WEIGHTS_COPY,
                 device: int = 0, ctx=None, op: int = jg.JG_OP_XWT, tail: int = jg.JG_TAIL_SPLIT,
                 dtype: int = jg.JG_F32, accumulate: int = jg.JG_ACC_LEVELS):
        if not torch.cuda.is_available():
            raise RuntimeError("JigsawLinear needs a GPU: the HIP library has no CPU fallback")
        self.M, self.K, self.N, self.ways, self.bias, self.op = M, K, N, ways, bias, op
        self.x_shape = (K, M) if op == jg.JG_OP_XTW else (M, K)
        self.w_shape = (N, K) if op == jg.JG_OP_XWT else (K, N)
        self.dev = torch.device("cuda", device)
        self._own_ctx = ctx is None
        self.stream = torch.cuda.current_stream(self.dev)
        self.ctx = ctx if ctx is not None else jg.jg_init(device, self.stream.cuda_stream)
        self.dtype = dtype
        self.plan = jg.jg_plan_create(self.ctx, M, K, N, ways, bias, combine, weights, op, dtype=dtype, tail=tail,
                                      accumulate=accumulate)
        q = lambda what, r=0: jg.jg_plan_query(self.plan, what, r)
        f32 = dict(dtype=torch.float32, device=self.dev)
        if dtype == jg.JG_F32:
            self.x = [torch.empty((q(jg.JG_Q_X_ROWS, r), q(jg.JG_Q_X_COLS, r)), **f32) for r in range(ways)]
            self.w = [torch.empty((q(jg.JG_Q_W_ROWS, r), q(jg.JG_Q_W_COLS, r)), **f32) for r in range(ways)]
        else:
            # rows are padded by the library (whole 128-byte lines per plane): the row length comes from the byte count
            b16 = dict(dtype=torch.bfloat16, device=self.dev)
            # (the transposed layer's shards are stored contraction-major: one row per column of the block)
            rowlen = lambda nbytes, rows: nbytes // (2 * rows)
            xrows, wrows = ((jg.JG_Q_X_COLS, jg.JG_Q_W_COLS) if op == jg.JG_OP_XTW else (jg.JG_Q_X_ROWS, jg.JG_Q_W_ROWS))
            self.x = [torch.empty((q(xrows, r), rowlen(q(jg.JG_Q_X_SHARD_BYTES, r), q(xrows, r))), **b16)
                      for r in range(ways)]
            self.w = [torch.empty((q(wrows, r), rowlen(q(jg.JG_Q_W_SHARD_BYTES, r), q(wrows, r))), **b16)
                      for r in range(ways)]
        self.y = [torch.empty((q(jg.JG_Q_Y_ROWS, r), q(jg.JG_Q_Y_COLS, r)), **f32) for r in range(ways)]
        self.b = [torch.empty((q(jg.JG_Q_B_LEN, r),), **f32) for r in range(ways)] if bias else None
        self.ws_bytes = q(jg.JG_Q_WORKSPACE_BYTES)
        self.ws = torch.empty((max(self.ws_bytes, 1),), dtype=torch.uint8, device=self.dev)

    # -- data movement ---------------------------------------------------------
    def shard(self, X=None, W=None, b=None):
        """Split global device tensors into the per-rank shards (jg_shard)."""
        if X is not None:
            assert X.is_cuda and X.dtype == torch.float32 and X.shape == self.x_shape and X.stride(1) == 1
            jg.jg_shard(self.plan, jg.JG_T_X, X.data_ptr(), X.stride(0), [t.data_ptr() for t in self.x])
        if W is not None:
            assert W.is_cuda and W.dtype == torch.float32 and W.shape == self.w_shape and W.stride(1) == 1
            jg.jg_shard(self.plan, jg.JG_T_W, W.data_ptr(), W.stride(0), [t.data_ptr() for t in self.w])
        if b is not None:
            assert self.bias and b.is_cuda and b.dtype == torch.float32 and b.shape == (self.N,)
            jg.jg_shard(self.plan, jg.JG_T_B, b.data_ptr(), self.N, [t.data_ptr() for t in self.b])

    def shard_patches(self, field, p: int):
        """X shards straight from a (C, H, W) field: the patch encoder's input (jg_shard_patches)."""
        assert field.is_cuda and field.dtype == torch.float32 and field.dim() == 3 and field.is_contiguous()
        C, H, W = field.shape
        jg.jg_shard_patches(self.plan, field.data_ptr(), C, H, W, p, [t.data_ptr() for t in self.x])

    def gather_patches(self, C: int, H: int, W: int, p: int, out=None):
        """(C, H, W) field from the Y shards: the patch decoder's output (jg_gather_patches)."""
        if out is None:
            out = torch.empty((C, H, W), dtype=torch.float32, device=self.dev)
        jg.jg_gather_patches(self.plan, [t.data_ptr() for t in self.y], out.data_ptr(), C, H, W, p)
        return out

    def forward(self, residual=None, activation: int = jg.JG_ACT_NONE):
        """Y_r = act(X W^T + b)_r (+ residual_r); ``residual``: per-rank tensors shaped like the Y shards."""
        if residual is None and activation == jg.JG_ACT_NONE:
            key = tuple(t.data_ptr() for t in self.x + self.w + self.y) + (self.ws.data_ptr(),)
            if getattr(self, "_fwd_key", None) != key:      # the shard buffers' addresses, marshalled once
                self._fwd_key = key
                self._fwd_args = (jg.ptr_array([t.data_ptr() for t in self.x]), jg.ptr_array([t.data_ptr() for t in self.w]),
                                  jg.ptr_array([t.data_ptr() for t in self.b]) if self.bias else None,
                                  jg.ptr_array([t.data_ptr() for t in self.y]),
                                  self.ws.data_ptr() if self.ws_bytes else None, self.ws_bytes)
            jg.jg_linear_forward(self.plan, *self._fwd_args)
            return
        if residual is not None:
            assert len(residual) == self.ways and all(r.shape == y.shape and r.is_contiguous()
                                                      for r, y in zip(residual, self.y))
        jg.jg_linear_forward_ex(self.plan, [t.data_ptr() for t in self.x], [t.data_ptr() for t in self.w],
                                [t.data_ptr() for t in self.b] if self.bias else None,
                                [t.data_ptr() for t in residual] if residual is not None else None, activation,
                                [t.data_ptr() for t in self.y],
                                self.ws.data_ptr() if self.ws_bytes else None, self.ws_bytes)

    def layernorm(self, gamma=None, beta=None, eps: float = 1e-5, out=None):
        """Layer norm of the X shards over each rank's channels (jg_layernorm_forward); ``gamma`` / ``beta``
        are device vectors over all channels of X.  Writes ``out`` (per-rank tensors shaped like the X
        shards; default: in place) and returns it."""
        C = self.x_shape[1]
        for v in (gamma, beta):
            assert v is None or (v.is_cuda and v.dtype == torch.float32 and v.shape == (C,) and v.is_contiguous())
        out = self.x if out is None else out
        assert len(out) == self.ways and all(o.shape == x.shape and o.is_contiguous() for o, x in zip(out, self.x))
        jg.jg_layernorm_forward(self.plan, [t.data_ptr() for t in self.x],
                                gamma.data_ptr() if gamma is not None else None,
                                beta.data_ptr() if beta is not None else None, eps, [t.data_ptr() for t in out])
        return out

    def gather(self, out=None):
        if out is None:
            out = torch.empty((self.M, self.N), dtype=torch.float32, device=self.dev)
        jg.jg_gather(self.plan, [t.data_ptr() for t in self.y], out.data_ptr(), out.stride(0))
        return out

    # -- backward ---------------------------------------------------------------
    def alloc_backward(self):
        """Shard tensors for dY (like Y), dX (like X), dW (like W) and the backward workspace.  A reduced-precision
        plan's backward reads FP32 copies of X and W (``x32`` / ``w32``, filled by ``shard``) and writes FP32 dX, dW."""
        if getattr(self, "dy", None) is None:
            q = self.query
            self.dy = [torch.empty_like(t) for t in self.y]
            if self.dtype == jg.JG_F32:
                self.x32, self.w32 = self.x, self.w
            else:
                f32 = dict(dtype=torch.float32, device=self.dev)
                self.x32 = [torch.empty((q(jg.JG_Q_X_ROWS, r), q(jg.JG_Q_X_COLS, r)), **f32) for r in range(self.ways)]
                self.w32 = [torch.empty((q(jg.JG_Q_W_ROWS, r), q(jg.JG_Q_W_COLS, r)), **f32) for r in range(self.ways)]
            self.dx = [torch.empty_like(t) for t in self.x32]
            self.dw = [torch.empty_like(t) for t in self.w32]
            self.bw_ws_bytes = self.query(jg.JG_Q_BACKWARD_WORKSPACE_BYTES)
            self.bw_ws = torch.empty((max(self.bw_ws_bytes, 1),), dtype=torch.uint8, device=self.dev)

    def shard_dy(self, dY):
        assert dY.is_cuda and dY.dtype == torch.float32 and dY.shape == (self.M, self.N) and dY.stride(1) == 1
        self.alloc_backward()
        jg.jg_shard(self.plan, jg.JG_T_Y, dY.data_ptr(), dY.stride(0), [t.data_ptr() for t in self.dy])

    def shard_master(self, X=None, W=None):
        """FP32 copies of X and W for the backward of a reduced-precision plan (JG_T_X_F32 / JG_T_W_F32 shards)."""
        self.alloc_backward()
        if X is not None:
            jg.jg_shard(self.plan, jg.JG_T_X_F32, X.data_ptr(), X.stride(0), [t.data_ptr() for t in self.x32])
        if W is not None:
            jg.jg_shard(self.plan, jg.JG_T_W_F32, W.data_ptr(), W.stride(0), [t.data_ptr() for t in self.w32])

    def backward(self):
        self.alloc_backward()
        jg.jg_linear_backward(self.plan, [t.data_ptr() for t in self.x32], [t.data_ptr() for t in self.w32],
                              [t.data_ptr() for t in self.dy], [t.data_ptr() for t in self.dx],
                              [t.data_ptr() for t in self.dw],
                              self.bw_ws.data_ptr() if self.bw_ws_bytes else None, self.bw_ws_bytes)

    def bias_backward(self):
        """db shards (shaped like the bias shards) = column sums of the dY shards (jg_bias_backward)."""
        self.alloc_backward()
        if getattr(self, "db", None) is None:
            self.db = [torch.empty((self.query(jg.JG_Q_B_LEN, r),), dtype=torch.float32, device=self.dev)
                       for r in range(self.ways)]
        if getattr(self, "db_ws", None) is None:
            self.db_ws_bytes = self.query(jg.JG_Q_BIAS_BACKWARD_WORKSPACE_BYTES)
            self.db_ws = torch.empty((max(self.db_ws_bytes, 8),), dtype=torch.uint8, device=self.dev)
        jg.jg_bias_backward(self.plan, [t.data_ptr() for t in self.dy], [t.data_ptr() for t in self.db],
                            self.db_ws.data_ptr() if self.db_ws_bytes else None, self.db_ws_bytes)
        return self.db

    def gather_dx(self):
        out = torch.empty(self.x_shape, dtype=torch.float32, device=self.dev)
        jg.jg_gather_as(self.plan, jg.JG_T_X_F32, [t.data_ptr() for t in self.dx], out.data_ptr(), out.stride(0))
        return out

    def gather_dw(self):
        out = torch.empty(self.w_shape, dtype=torch.float32, device=self.dev)
        jg.jg_gather_as(self.plan, jg.JG_T_W_F32, [t.data_ptr() for t in self.dw], out.data_ptr(), out.stride(0))
        return out

    def query(self, what: int, rank: int = 0) -> int:
        return jg.jg_plan_query(self.plan, what, rank)

    def close(self):
        if self.plan:
            jg.jg_plan_destroy(self.plan)
            self.plan = None
        if self._own_ctx and self.ctx:
            jg.jg_free(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


class JigsawMLP:
    """One mixing MLP with its skip connection on Jigsaw shards: H = gelu(X W1^T + b1), Y = X + H W2^T + b2.

    X and Y are (M, C), W1 is (Hd, C), W2 is (C, Hd).  Two JigsawLinear holders share one context; the
    second reads the first one's output shards in place (``jg_mlp_forward``).  ``dtype = JG_BF16 /
    JG_BF16X3``: mixed precision - the weight shards are bfloat16, X, H and Y stay FP32 and each layer rounds
    its input into the workspace.
    """

    def __init__(self, M: int, C: int, Hd: int, ways: int, device: int = 0, ctx=None, tail: int = jg.JG_TAIL_SPLIT,
                 dtype: int = jg.JG_F32, accumulate: int = jg.JG_ACC_LEVELS):
        self.first = JigsawLinear(M, C, Hd, ways, bias=True, device=device, ctx=ctx, tail=tail, dtype=dtype,
                                  accumulate=accumulate)
        self.second = JigsawLinear(M, Hd, C, ways, bias=True, device=device, ctx=self.first.ctx, tail=tail, dtype=dtype,
                                   accumulate=accumulate)
        self.dtype = dtype
        if dtype == jg.JG_F32:
            self.xin = self.first.x
        else:       # FP32 activations, partitioned like X (the holders' bfloat16 X shards are not used)
            q = self.first.query
            self.xin = [torch.empty((q(jg.JG_Q_X_ROWS, r), q(jg.JG_Q_X_COLS, r)), dtype=torch.float32,
                                    device=self.first.dev) for r in range(ways)]
            self.first.x = None
        self.second.x = self.first.y        # H_r is consumed where it was produced
        self.M, self.C, self.Hd, self.ways = M, C, Hd, ways
        self.ctx = self.first.ctx
        chain = [L.query(jg.JG_Q_CHAIN_WORKSPACE_BYTES) for L in (self.first, self.second)]
        self.ws_bytes = max(chain) if dtype == jg.JG_F32 else sum(chain)
        self.ws = max((self.first.ws, self.second.ws), key=lambda t: t.numel())
        if self.ws.numel() < self.ws_bytes:
            self.first.ws = self.second.ws = None
            self.ws = torch.empty((self.ws_bytes,), dtype=torch.uint8, device=self.first.dev)

    def shard(self, X=None, W1=None, b1=None, W2=None, b2=None):
        if X is not None:
            assert X.is_cuda and X.dtype == torch.float32 and X.shape == (self.M, self.C) and X.stride(1) == 1
            jg.jg_shard(self.first.plan, jg.JG_T_X_F32, X.data_ptr(), X.stride(0), [t.data_ptr() for t in self.xin])
        self.first.shard(None, W1, b1)
        self.second.shard(None, W2, b2)
        if self.dtype != jg.JG_F32 and getattr(self, "keep_masters", False):
            # mixed-precision training keeps the FP32 weights: the backward reads them
            self.first.shard_master(None, W1)
            self.second.shard_master(None, W2)

    def forward(self):
        f, s = self.first, self.second
        jg.jg_mlp_forward(f.plan, s.plan, [t.data_ptr() for t in self.xin], [t.data_ptr() for t in f.w],
                          [t.data_ptr() for t in f.b], [t.data_ptr() for t in s.w], [t.data_ptr() for t in s.b],
                          [t.data_ptr() for t in f.y], [t.data_ptr() for t in s.y],
                          self.ws.data_ptr() if self.ws_bytes else None, self.ws_bytes)

    def gather_h(self):
        return self.first.gather()

    def gather(self):
        return self.second.gather()

    # -- backward --------------------------------------------------------------------
    def master_weights(self):
        """(W1 shards, W2 shards) in FP32: the plans' own for FP32 plans, the kept masters in mixed precision
        (set ``keep_masters = True`` before ``shard``)."""
        f, s = self.first, self.second
        if self.dtype == jg.JG_F32:
            return f.w, s.w
        assert getattr(f, "w32", None) is not None, "mixed-precision backward: set keep_masters before shard()"
        return f.w32, s.w32

    def backward_workspace_bytes(self):
        f, s = self.first, self.second
        up = lambda n: (n + 255) // 256 * 256
        recompute = f.query(jg.JG_Q_CHAIN_WORKSPACE_BYTES)
        if self.dtype != jg.JG_F32:
            recompute += self.ways * up(f.query(jg.JG_Q_W_SHARD_BYTES))
        return max(recompute, f.query(jg.JG_Q_BACKWARD_WORKSPACE_BYTES), s.query(jg.JG_Q_BACKWARD_WORKSPACE_BYTES),
                   f.query(jg.JG_Q_NORM_BACKWARD_WORKSPACE_BYTES))

    def backward(self, dY):
        """Gradients for an incoming gradient dY (M, C), after forward(): jg_mlp_backward.  The shards of A, dH, dA,
        dX, dW1, db1, dW2, db2 are kept on the holder (``self.grads``).  Mixed precision: the same call on the FP32
        activations and master weights, every product's operands rounded as in the forward."""
        f, s = self.first, self.second
        assert dY.is_cuda and dY.dtype == torch.float32 and dY.shape == (self.M, self.C)
        w1, w2 = self.master_weights()
        if getattr(self, "grads", None) is None:
            like = lambda ts: [torch.empty_like(t) for t in ts]
            self.grads = dict(dy=like(s.y), a=like(f.y), dh=like(f.y), da=like(f.y), dx=like(self.xin), dw1=like(w1),
                              db1=like(f.b), dw2=like(w2), db2=like(s.b))
            need = self.backward_workspace_bytes()
            self.bw_ws = torch.empty((max(need, 1),), dtype=torch.uint8, device=f.dev)
            self.bw_ws_bytes = need
        g = self.grads
        p = lambda ts: [t.data_ptr() for t in ts]
        jg.jg_shard(s.plan, jg.JG_T_Y, dY.data_ptr(), dY.stride(0), p(g["dy"]))
        jg.jg_mlp_backward(f.plan, s.plan, p(self.xin), p(w1), p(f.b), p(w2), p(f.y), p(g["dy"]), p(g["a"]), p(g["dh"]),
                           p(g["da"]), p(g["dx"]), p(g["dw1"]), p(g["db1"]), p(g["dw2"]), p(g["db2"]),
                           self.bw_ws.data_ptr() if self.bw_ws_bytes else None, self.bw_ws_bytes)

    def gather_grad(self, name: str):
        """A gradient (or kept intermediate) of backward() as a global matrix: 'a', 'dh', 'da' (M, Hd), 'dx' (M, C),
        'dw1' (Hd, C), 'dw2' (C, Hd); 'db1', 'db2' as global vectors."""
        f, s, g = self.first, self.second, self.grads
        p = lambda ts: [t.data_ptr() for t in ts]
        dev = f.dev
        if name in ("a", "dh", "da"):
            out = torch.empty((self.M, self.Hd), dtype=torch.float32, device=dev)
            jg.jg_gather_as(f.plan, jg.JG_T_Y, p(g[name]), out.data_ptr(), out.stride(0))
        elif name in ("dx", "dxn"):
            out = torch.empty((self.M, self.C), dtype=torch.float32, device=dev)
            jg.jg_gather_as(f.plan, jg.JG_T_X_F32, p(g[name]), out.data_ptr(), out.stride(0))
        elif name in ("dw1", "dw2"):
            L = f if name == "dw1" else s
            out = torch.empty(L.w_shape, dtype=torch.float32, device=dev)
            jg.jg_gather_as(L.plan, jg.JG_T_W_F32, p(g[name]), out.data_ptr(), out.stride(0))
        else:       # bias gradients: rank r holds the slice of column half r % 2 (replicated in the 4-way form)
            L = f if name == "db1" else s
            parts = g[name][:1] if self.ways == 1 else g[name][:2]
            out = torch.cat(parts)
        return out

    def close(self):
        self.second.close()
        self.first.close()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


class JigsawMixing(JigsawMLP):
    """Channel-mixing half of a mixing block: Xn = layernorm(X), H = gelu(Xn W1^T + b1), Y = X + H W2^T + b2
    (``jg_mixing_forward``).  ``gamma`` / ``beta``: device vectors of length C."""

    def __init__(self, M: int, C: int, Hd: int, ways: int, device: int = 0, ctx=None, tail: int = jg.JG_TAIL_SPLIT,
                 eps: float = 1e-5, dtype: int = jg.JG_F32, accumulate: int = jg.JG_ACC_LEVELS):
        super().__init__(M, C, Hd, ways, device=device, ctx=ctx, tail=tail, dtype=dtype, accumulate=accumulate)
        self.eps = eps
        self.xn = [torch.empty_like(t) for t in self.xin]
        self.gamma = self.beta = None

    def shard(self, X=None, gamma=None, beta=None, W1=None, b1=None, W2=None, b2=None):
        super().shard(X, W1, b1, W2, b2)
        for v in (gamma, beta):
            assert v is None or (v.is_cuda and v.dtype == torch.float32 and v.shape == (self.C,) and v.is_contiguous())
        self.gamma, self.beta = gamma, beta

    def forward(self):
        f, s = self.first, self.second
        p = lambda ts: [t.data_ptr() for t in ts]
        jg.jg_mixing_forward(f.plan, s.plan, p(self.xin), self.gamma.data_ptr() if self.gamma is not None else None,
                             self.beta.data_ptr() if self.beta is not None else None, self.eps, p(f.w), p(f.b),
                             p(s.w), p(s.b), p(self.xn), p(f.y), p(s.y),
                             self.ws.data_ptr() if self.ws_bytes else None, self.ws_bytes)

    def gather_xn(self):
        out = torch.empty((self.M, self.C), dtype=torch.float32, device=self.first.dev)
        jg.jg_gather_as(self.first.plan, jg.JG_T_X_F32, [t.data_ptr() for t in self.xn], out.data_ptr(), out.stride(0))
        return out

    def backward(self, dY=None, dy_shards=None):
        """Gradients of the block for an incoming gradient dY (M, C), after forward(): jg_mixing_backward.  Beside
        the MLP's (JigsawMLP.backward) the holder keeps 'dxn' shards and the global vectors ``dgamma`` / ``dbeta``.
        ``dy_shards``: the gradient already on shards partitioned like X_r (another block's 'dx'), instead of dY."""
        f, s = self.first, self.second
        assert (dY is None) != (dy_shards is None)
        assert dY is None or (dY.is_cuda and dY.dtype == torch.float32 and dY.shape == (self.M, self.C))
        w1, w2 = self.master_weights()
        if getattr(self, "grads", None) is None:
            like = lambda ts: [torch.empty_like(t) for t in ts]
            self.grads = dict(dy=like(s.y), a=like(f.y), dh=like(f.y), da=like(f.y), dxn=like(self.xin),
                              dx=like(self.xin), dw1=like(w1), db1=like(f.b), dw2=like(w2), db2=like(s.b))
            self.dgamma = torch.empty((self.C,), dtype=torch.float32, device=f.dev)
            self.dbeta = torch.empty((self.C,), dtype=torch.float32, device=f.dev)
            need = self.backward_workspace_bytes()
            self.bw_ws = torch.empty((need,), dtype=torch.uint8, device=f.dev)
            self.bw_ws_bytes = need
        g = self.grads
        p = lambda ts: [t.data_ptr() for t in ts]
        dy = g["dy"] if dy_shards is None else dy_shards
        if dy_shards is None:
            jg.jg_shard(s.plan, jg.JG_T_Y, dY.data_ptr(), dY.stride(0), p(dy))
        jg.jg_mixing_backward(f.plan, s.plan, p(self.xin), self.gamma.data_ptr() if self.gamma is not None else None,
                              self.eps, p(self.xn), p(w1), p(f.b), p(w2), p(f.y), p(dy), p(g["a"]), p(g["dh"]),
                              p(g["da"]), p(g["dxn"]), p(g["dx"]), p(g["dw1"]), p(g["db1"]), p(g["dw2"]), p(g["db2"]),
                              self.dgamma.data_ptr(), self.dbeta.data_ptr(), self.bw_ws.data_ptr(), self.bw_ws_bytes)


class JigsawTokenMixing:
    """Token-mixing half of a mixing block: Xn = layernorm(X), H = gelu(Xn^T W1 + b1), Y = X + W2 H^T + b2 1^T
    (``jg_token_mixing_forward``).  X and Y are (T, C), W1 and W2 are (T, D), b1 is (D,), b2 is (T,), gamma and beta
    are (C,).  The first holder is the transposed layer (X^T W), the second a plain layer in which W2 stands where
    the activations do and H where the weights do; nothing is transposed in memory."""

    def __init__(self, T: int, C: int, D: int, ways: int, device: int = 0, ctx=None, tail: int = jg.JG_TAIL_SPLIT,
                 eps: float = 1e-5, dtype: int = jg.JG_F32, accumulate: int = jg.JG_ACC_LEVELS):
        """``dtype = JG_BF16 / JG_BF16X3``: mixed precision - X, Xn, H and Y stay FP32, the two products read
        bfloat16 roundings (W1 and W2 rounded when sharded, Xn and H by the chain, into the workspace)."""
        self.first = JigsawLinear(C, T, D, ways, bias=True, device=device, ctx=ctx, op=jg.JG_OP_XTW, tail=tail,
                                  dtype=dtype, accumulate=accumulate)
        self.second = JigsawLinear(T, D, C, ways, bias=False, device=device, ctx=self.first.ctx, tail=tail, dtype=dtype,
                                   accumulate=accumulate)
        self.second.w = self.first.y        # H_r is the second layer's weight shard, read where it was produced
        self.T, self.C, self.D, self.ways, self.eps, self.dtype = T, C, D, ways, eps, dtype
        self.ctx = self.first.ctx
        q = self.first.query
        if dtype == jg.JG_F32:
            self.xin = self.first.x
        else:                               # the activations enter in FP32; only the products' operands are rounded
            self.xin = [torch.empty((q(jg.JG_Q_X_ROWS, r), q(jg.JG_Q_X_COLS, r)), dtype=torch.float32,
                                    device=self.first.dev) for r in range(ways)]
            self.first.x = None
        self.xn = [torch.empty_like(t) for t in self.xin]
        self.gamma = self.beta = self.b2 = None
        up = lambda n: (n + 255) // 256 * 256
        self.ws_bytes = max(self.first.ws_bytes, self.second.ws_bytes) + q(jg.JG_Q_X_F32_SHARDS_BYTES)
        if dtype != jg.JG_F32:
            self.ws_bytes += ways * (up(q(jg.JG_Q_X_SHARD_BYTES)) + up(self.second.query(jg.JG_Q_W_SHARD_BYTES)))
        self.first.ws = self.second.ws = None
        self.ws = torch.empty((max(self.ws_bytes, 1),), dtype=torch.uint8, device=self.first.dev)

    def shard(self, X=None, gamma=None, beta=None, W1=None, b1=None, W2=None, b2=None):
        if X is not None:
            assert X.is_cuda and X.dtype == torch.float32 and X.shape == (self.T, self.C) and X.stride(1) == 1
            jg.jg_shard(self.first.plan, jg.JG_T_X_F32, X.data_ptr(), X.stride(0), [t.data_ptr() for t in self.xin])
        self.first.shard(None, W1, b1)
        if self.dtype != jg.JG_F32 and getattr(self, "keep_masters", False):
            # mixed-precision training keeps the FP32 weights: the backward reads them
            self.first.shard_master(None, W1)
            self.second.shard_master(W2, None)
        if W2 is not None:      # W2 takes the place of the second layer's activations
            assert W2.is_cuda and W2.dtype == torch.float32 and W2.shape == (self.T, self.D) and W2.stride(1) == 1
            jg.jg_shard(self.second.plan, jg.JG_T_X, W2.data_ptr(), W2.stride(0), [t.data_ptr() for t in self.second.x])
        for v, n in ((gamma, self.C), (beta, self.C), (b2, self.T)):
            assert v is None or (v.is_cuda and v.dtype == torch.float32 and v.shape == (n,) and v.is_contiguous())
        self.gamma, self.beta, self.b2 = gamma, beta, b2

    def forward(self):
        f, s = self.first, self.second
        p = lambda ts: [t.data_ptr() for t in ts]
        opt = lambda v: v.data_ptr() if v is not None else None
        jg.jg_token_mixing_forward(f.plan, s.plan, p(self.xin), opt(self.gamma), opt(self.beta), self.eps, p(f.w), p(f.b),
                                   p(s.x), opt(self.b2), p(self.xn), p(f.y), p(s.y), self.ws.data_ptr(), self.ws_bytes)

    def gather_xn(self):
        out = torch.empty((self.T, self.C), dtype=torch.float32, device=self.first.dev)
        jg.jg_gather_as(self.first.plan, jg.JG_T_X_F32, [t.data_ptr() for t in self.xn], out.data_ptr(), out.stride(0))
        return out

    def backward(self, dY=None, dy_shards=None):
        """Gradients of the block for an incoming gradient dY (T, C), after forward(): jg_token_mixing_backward.  The
        shards of A, dH, dA, dXn, dX, dW1, db1, dW2 are kept on the holder (``self.grads``), ``db2`` (T,), ``dgamma``
        and ``dbeta`` (C,) as global vectors.  ``dy_shards``: the gradient already on shards partitioned like X_r
        (another block's 'dx'), instead of dY."""
        f, s = self.first, self.second
        assert (dY is None) != (dy_shards is None)
        assert dY is None or (dY.is_cuda and dY.dtype == torch.float32 and dY.shape == (self.T, self.C))
        if getattr(self, "grads", None) is None:
            like = lambda ts: [torch.empty_like(t) for t in ts]
            w1, w2 = self.master_weights()
            self.grads = dict(dy=like(s.y), a=like(f.y), dh=like(f.y), da=like(f.y), dxn=like(self.xin),
                              dx=like(self.xin), dw1=like(w1), db1=like(f.b), dw2=like(w2))
            vec = lambda n: torch.empty((n,), dtype=torch.float32, device=f.dev)
            self.db2, self.dgamma, self.dbeta = vec(self.T), vec(self.C), vec(self.C)
            up = lambda n: (n + 255) // 256 * 256
            recompute = f.query(jg.JG_Q_CHAIN_WORKSPACE_BYTES)
            if self.dtype != jg.JG_F32:
                recompute += self.ways * up(f.query(jg.JG_Q_W_SHARD_BYTES))
            need = max(recompute, f.query(jg.JG_Q_BACKWARD_WORKSPACE_BYTES),
                       s.query(jg.JG_Q_BACKWARD_WORKSPACE_BYTES), f.query(jg.JG_Q_NORM_BACKWARD_WORKSPACE_BYTES))
            self.bw_ws = torch.empty((need,), dtype=torch.uint8, device=f.dev)
            self.bw_ws_bytes = need
        g = self.grads
        p = lambda ts: [t.data_ptr() for t in ts]
        dy = g["dy"] if dy_shards is None else dy_shards
        if dy_shards is None:
            jg.jg_shard(s.plan, jg.JG_T_Y, dY.data_ptr(), dY.stride(0), p(dy))
        w1, w2 = self.master_weights()
        jg.jg_token_mixing_backward(f.plan, s.plan, p(self.xin), self.gamma.data_ptr() if self.gamma is not None else None,
                                    self.eps, p(self.xn), p(w1), p(f.b), p(w2), p(f.y), p(dy), p(g["a"]),
                                    p(g["dh"]), p(g["da"]), p(g["dxn"]), p(g["dx"]), p(g["dw1"]), p(g["db1"]),
                                    p(g["dw2"]), self.db2.data_ptr(), self.dgamma.data_ptr(), self.dbeta.data_ptr(),
                                    self.bw_ws.data_ptr(), self.bw_ws_bytes)

    def master_weights(self):
        """(W1 shards, W2 shards) in FP32: the plans' own for FP32 plans, the kept masters in mixed precision
        (set ``keep_masters = True`` before ``shard``)."""
        f, s = self.first, self.second
        if self.dtype == jg.JG_F32:
            return f.w, s.x
        assert getattr(f, "w32", None) is not None, "mixed-precision backward: set keep_masters before shard()"
        return f.w32, s.x32

    def gather_grad(self, name: str):
        """A gradient (or kept intermediate) of backward() as a global matrix: 'a', 'dh', 'da' (C, D), 'dx', 'dxn'
        (T, C), 'dw1', 'dw2' (T, D); 'db1' as a global vector (D,)."""
        f, s, g = self.first, self.second, self.grads
        p = lambda ts: [t.data_ptr() for t in ts]
        if name == "db1":       # rank r holds the slice of column half r % 2 (replicated in the 4-way form)
            return torch.cat(g[name][:1] if self.ways == 1 else g[name][:2])
        plan, which, shape = {"a": (f, jg.JG_T_Y, (self.C, self.D)), "dh": (f, jg.JG_T_Y, (self.C, self.D)),
                              "da": (f, jg.JG_T_Y, (self.C, self.D)), "dx": (f, jg.JG_T_X_F32, (self.T, self.C)),
                              "dxn": (f, jg.JG_T_X_F32, (self.T, self.C)), "dw1": (f, jg.JG_T_W_F32, (self.T, self.D)),
                              "dw2": (s, jg.JG_T_X_F32, (self.T, self.D))}[name]
        out = torch.empty(shape, dtype=torch.float32, device=f.dev)
        jg.jg_gather_as(plan.plan, which, p(g[name]), out.data_ptr(), out.stride(0))
        return out

    def gather_h(self):
        return self.first.gather()

    def gather(self):
        return self.second.gather()

    def close(self):
        self.second.close()
        self.first.close()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


class JigsawMixerBlock:
    """One mixing block (Sec. 3): the token-mixing half followed by the channel-mixing half, each with its layer norm
    and skip connection, on Jigsaw shards.  X and Y are (T, C).  The token half leaves its output partitioned like
    X, which is how the channel half reads its input: the second half works on the first one's output shards in
    place."""

    def __init__(self, T: int, C: int, Dt: int, Dc: int, ways: int, device: int = 0, ctx=None,
                 tail: int = jg.JG_TAIL_SPLIT, eps: float = 1e-5, dtype: int = jg.JG_F32, keep_masters: bool = False,
                 accumulate: int = jg.JG_ACC_LEVELS):
        """``dtype = JG_BF16 / JG_BF16X3``: both halves in mixed precision (FP32 activations between them);
        ``keep_masters``: also keep the FP32 weights on shards, which the mixed-precision backward reads."""
        self.token = JigsawTokenMixing(T, C, Dt, ways, device=device, ctx=ctx, tail=tail, eps=eps, dtype=dtype,
                                       accumulate=accumulate)
        self.channel = JigsawMixing(T, C, Dc, ways, device=device, ctx=self.token.ctx, tail=tail, eps=eps, dtype=dtype,
                                    accumulate=accumulate)
        self.token.keep_masters = self.channel.keep_masters = keep_masters
        self.channel.xin = self.token.second.y
        if dtype == jg.JG_F32:
            self.channel.first.x = self.token.second.y
        self.T, self.C, self.ways = T, C, ways
        self.ctx = self.token.ctx

    def shard(self, X=None, token=None, channel=None):
        """token: dict(gamma, beta, W1, b1, W2, b2) of the token half; channel: the same names for the channel half."""
        if X is not None or token:
            self.token.shard(X, **(token or {}))
        if channel:
            self.channel.shard(None, **channel)

    def forward(self):
        self.token.forward()
        self.channel.forward()

    def backward(self, dY):
        """Gradients of the whole block for an incoming gradient dY (T, C), after forward(): the channel half's
        backward, then the token half's on the channel half's dX shards in place (they are partitioned as the token
        half's dY).  The gradients stay on the two halves (``self.channel`` / ``self.token``: grads, dgamma, dbeta,
        db2); the block's dX is the token half's."""
        self.channel.backward(dY)
        self.token.backward(dy_shards=self.channel.grads["dx"])

    def gather_dx(self):
        return self.token.gather_grad("dx")

    def gather_token_output(self):
        return self.token.gather()

    def gather(self):
        return self.channel.gather()

    def close(self):
        self.channel.close()
        self.token.close()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
