"""Buffers of one MoE verify layer plus the five library calls in order.  No arithmetic here:
the class only owns the output / scratch tensors (allocated once) and marshals arguments."""
from __future__ import annotations

import torch

from . import binding as B


class MoEVerifyLayer:
    """route -> permute -> grouped SwiGLU -> combine on preallocated buffers.

    T tokens = B sequences x (gamma+1) positions (the tokens one verification pass scores).
    """

    def __init__(self, T, d_model, d_ff, E, k, dtype, device="cuda", renorm=True,
                 fuse_gather=True):
        """fuse_gather: moe_permute writes indices only and the gate/up GEMM gathers token rows
        itself (moe_expert_up_swiglu_gather); False materialises x_perm first."""
        self.T, self.d, self.f, self.E, self.k = T, d_model, d_ff, E, k
        self.dtype, self.renorm = dtype, renorm
        self.fuse_gather = fuse_gather and T * d_model * (4 if dtype == torch.float32 else 2) < 2 ** 32
        P = T * k
        dev = torch.device(device)
        i32 = dict(dtype=torch.int32, device=dev)
        self.topk_idx = torch.empty((T, k), **i32)
        self.topk_w = torch.empty((T, k), dtype=torch.float32, device=dev)
        self.expert_offsets = torch.empty((E + 1,), **i32)
        self.row_src = torch.empty((P,), **i32)
        self.row_of = torch.empty((P,), **i32)
        self.x_perm = torch.empty((P, d_model), dtype=dtype, device=dev)
        self.y_perm = torch.empty((P, d_model), dtype=dtype, device=dev)
        self.out = torch.empty((T, d_model), dtype=dtype, device=dev)
        self.h = torch.empty((P, d_ff), dtype=dtype, device=dev)
        self.h_packed = None                     # allocated on first use of packed weights
        self.x_packed = None

    # Which projections run on tile-packed operands (measured crossovers, average rows per
    # expert r = T*k/E): the packed gate/up kernel is ahead from r >= 48, and at any r when the
    # contraction is short (d_model < 4096, where the row-major alternative is the
    # register-staged kernel); the packed down kernel from r >= 96, or with d_ff < 4096.
    PACKED_UP_MIN_ROWS = 48
    PACKED_DOWN_MIN_ROWS = 96

    @classmethod
    def packed_plan(cls, n_pairs, E, d_model, d_ff):
        """(gate/up on packed operands?, down on packed operands?) for a batch of n_pairs
        (token, expert) pairs."""
        up = n_pairs >= cls.PACKED_UP_MIN_ROWS * E or d_model < 4096
        down = up and (n_pairs >= cls.PACKED_DOWN_MIN_ROWS * E or d_ff < 4096)
        return up, down

    @staticmethod
    def pack_weights(w_gate, w_up, w_down, stream=None):
        """One-time re-layout of the expert weights for the tile-packed kernels (bf16 only):
        returns the dict to pass as `packed=` to forward().  The row-major tensors stay valid and
        are still used whenever packed_plan() sends a projection to the row-major kernels."""
        out = {}
        for name, w in (("w_gate", w_gate), ("w_up", w_up), ("w_down", w_down)):
            wp = torch.empty_like(w)
            B.moe_pack_weights(w, wp, stream)
            out[name] = wp
        return out

    def forward(self, x, w_router, w_gate, w_up, w_down, bias=None, residual=None, out=None,
                stream=None, marks=None, draft_remap=None, packed=None):
        """Enqueues the layer.  `marks`, if given, is a sequence of six torch events recorded on
        `stream` before the router and after each of the five steps (route, permute, gate/up,
        down, combine): the benchmark's per-kernel times.  On the tile-packed path the permute
        step includes the gather of the token rows into tile-packed form.
        `draft_remap` ([E] int32 from moe_nearest_draft_expert) switches to the draft model's
        routing: selected experts that are not resident are replaced by their nearest draft
        expert, so only draft experts compute.
        `packed` (from pack_weights) lets the expert GEMMs run on tile-packed operands where
        packed_plan() says they are the faster ones (bf16 only)."""
        out = self.out if out is None else out
        up_packed = down_packed = False
        if packed is not None and self.dtype == torch.bfloat16 and self.fuse_gather:
            up_packed, down_packed = self.packed_plan(self.T * self.k, self.E, self.d, self.f)
        if marks is not None:
            marks[0].record(stream)
        if draft_remap is None:
            B.moe_route_topk(x, w_router, bias, self.k, self.renorm, self.topk_idx, self.topk_w,
                             stream)
        else:
            B.moe_route_topk_draft(x, w_router, bias, self.k, self.renorm, draft_remap,
                                   self.topk_idx, self.topk_w, stream)
        if marks is not None:
            marks[1].record(stream)
        B.moe_permute(x, self.topk_idx, self.E, None if self.fuse_gather else self.x_perm,
                      self.expert_offsets, self.row_src, self.row_of, stream)
        if up_packed:
            if self.x_packed is None:
                self.x_packed = torch.empty(
                    (B.moe_packed_h_bytes(self.T * self.k, self.d, self.E),), dtype=torch.uint8,
                    device=self.h.device)
            if down_packed and self.h_packed is None:
                self.h_packed = torch.empty(
                    (B.moe_packed_h_bytes(self.T * self.k, self.f, self.E),), dtype=torch.uint8,
                    device=self.h.device)
            # the data movement of the permute step, written once in the GEMM's own layout
            B.moe_permute_rows_packed(x, self.row_src, self.k, self.expert_offsets,
                                      self.T * self.k, self.x_packed, stream)
        if marks is not None:
            marks[2].record(stream)
        if up_packed:
            B.moe_expert_up_swiglu_packed(self.x_packed, self.expert_offsets, packed["w_gate"],
                                          packed["w_up"], self.T * self.k,
                                          self.h_packed if down_packed else self.h,
                                          not down_packed, stream)
        elif self.fuse_gather:
            B.moe_expert_up_swiglu_gather(x, self.row_src, self.k, self.expert_offsets, w_gate,
                                          w_up, self.h, stream)
        else:
            B.moe_expert_up_swiglu(self.x_perm, self.expert_offsets, w_gate, w_up, self.h, stream)
        if marks is not None:
            marks[3].record(stream)
        if down_packed:
            B.moe_expert_down_packed(self.h_packed, self.expert_offsets, packed["w_down"],
                                     self.y_perm, stream)
        else:
            B.moe_expert_down(self.h, self.expert_offsets, w_down, self.y_perm, stream)
        if marks is not None:
            marks[4].record(stream)
        B.moe_combine(self.y_perm, self.row_of, self.topk_w, residual, out, stream)
        if marks is not None:
            marks[5].record(stream)
        return out


class MoEVerifyStack:
    """n_layers x [RMSNorm -> MoE verify layer -> residual add] on one set of shared buffers.

    h_0 = x;  h_{l+1} = h_l + MoE_l(RMSNorm_l(h_l)).  The residual add is fused into
    moe_combine.  Layer weights stay resident in HBM (lists of per-layer tensors).
    """

    def __init__(self, T, d_model, d_ff, E, k, dtype, device="cuda", renorm=True, eps=1e-5):
        self.layer = MoEVerifyLayer(T, d_model, d_ff, E, k, dtype, device, renorm)
        self.eps = eps
        dev = torch.device(device)
        self.normed = torch.empty((T, d_model), dtype=dtype, device=dev)
        self.h = [torch.empty((T, d_model), dtype=dtype, device=dev) for _ in range(2)]

    def forward(self, x, layers, keep_hidden=False, stream=None, marks=None):
        """`layers`: list of dicts with gain, w_router, bias, w_gate, w_up, w_down.
        Returns the final hidden state (and, if keep_hidden, clones of every h_l).
        `marks`: six events recorded around the calls of the first layer (benchmark only)."""
        hidden = [x.clone()] if keep_hidden else None
        cur = x
        for li, L in enumerate(layers):
            nxt = self.h[li % 2]
            B.moe_rmsnorm(cur, L["gain"], self.eps, self.normed, stream)
            self.layer.forward(self.normed, L["w_router"], L["w_gate"], L["w_up"], L["w_down"],
                               L.get("bias"), residual=cur, out=nxt, stream=stream,
                               marks=marks if li == 0 else None)
            cur = nxt
            if keep_hidden:
                hidden.append(cur.clone())
        return (cur, hidden) if keep_hidden else cur


class GraphedStep:
    """One invocation of `fn(stream)` captured in a HIP graph and replayed with a single launch.

    `fn` must only enqueue library calls on preallocated buffers (MoEVerifyLayer.forward,
    MoEVerifyStack.forward without keep_hidden, spec_accept, ...): the library allocates nothing
    and records no memset nodes, so the captured graph is kernels only.  Inputs are read from the
    same tensors on every replay; refresh them in place (`x.copy_(...)`) between replays.
    Pays off where launch gaps matter: few-token configurations and the multi-layer stack
    (about 190 launches per step).
    """

    def __init__(self, fn, warmup=2):
        self.stream = torch.cuda.Stream()          # default priority
        self.stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(self.stream):
            for _ in range(warmup):                # one-time kernel attribute set-up happens here
                fn(self.stream)
        self.stream.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph, stream=self.stream):
            fn(self.stream)

    def replay(self):
        self.graph.replay()
