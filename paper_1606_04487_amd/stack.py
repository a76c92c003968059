"""A chain of convolution layers (conv -> ReLU -> optional 3x3/2 max-pool) run through the library.

This is the thin harness the tests and the bench use for the paper's CIFAR-style and
CaffeNet-style convolution phases (Sec. II-C: the "conv phase" of a CNN; Sec. IV-A: an engine is
a list of layers run forward and then in reverse).  It only sequences calls of the binding and
owns the device buffers; every arithmetic step runs in the library's kernels.

Memory plan (sized for one MI355X's 288 GB): every layer keeps its own forward workspace, so the
lowered matrix D-hat written by the forward pass is still there when the backward pass needs it
for the model gradient (the paper's "b_p = b": lower the whole batch once, Sec. III-B).  The
data-gradient workspace is shared by all layers.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B
from .workloads import ConvLayer


class ConvStack:
    def __init__(self, layers: Sequence[ConvLayer], dtype: int = B.F32, ceil_mode: bool = True,
                 skip_first_dgrad: bool = True, device: str = "cuda", fused: bool = True,
                 overlap_wgrad: bool = False, dy_rows: bool = True,
                 fuse_relu_dgrad: bool = True):
        self.layers = list(layers)
        self.dtype = dtype
        self.tdtype = B.torch_dtype(dtype)
        self.ceil_mode = ceil_mode
        self.skip_first_dgrad = skip_first_dgrad   # App. B: the first layer needs no data gradient
        self.device = device
        # overlap_wgrad = run every layer's model gradient on a second stream beside the data gradient of the
        # same layer (both only read dY of that layer; they write different tensors and use different
        # workspaces); the streams join before backward() returns
        self.side = torch.cuda.Stream(device=device) if overlap_wgrad else None
        # fused = let the library skip D-hat / dD-hat where it can (App. C: fusing lowering and GEMM);
        # the model gradient then reads its lowered operand straight from X (or lowers X itself where it
        # cannot) instead of finding D-hat cached by the forward pass
        extra = B.FLAG_FUSED if fused else 0
        # fully connected layers (whole-image windows) have few columns: split their reductions over the chip
        # (and take the explicit path, whose products on W and dY as they lie need no lowering there)
        self.desc = [B.conv_desc(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p, dtype,
                                 (B.FLAG_RELU if L.relu else 0) | (B.FLAG_SPLIT_K if L.Ho * L.Wo == 1 else extra))
                     for L in self.layers]
        self.dropout_seed = 1
        self.fwd_fused = [fused and B.conv_fused_supported(d, B.PASS_FORWARD) for d in self.desc]
        self.desc_wgrad = [d.with_flags((B.FLAG_FUSED if ff else B.FLAG_DHAT_CACHED) | (d.flags & B.FLAG_SPLIT_K))
                           for d, ff in zip(self.desc, self.fwd_fused)]
        # parameters: fp32 masters, velocity, gradients; bf16 copies of W for the bf16 passes
        self.W = [torch.zeros((L.F, L.C, L.k, L.k), dtype=torch.float32, device=device) for L in self.layers]
        self.b = [torch.zeros((L.F,), dtype=torch.float32, device=device) for L in self.layers]
        self.VW = [torch.zeros_like(w) for w in self.W]
        self.Vb = [torch.zeros_like(b) for b in self.b]
        self.dW = [torch.empty_like(w) for w in self.W]
        self.db = [torch.empty_like(b) for b in self.b]
        self.Wc = ([torch.zeros_like(w, dtype=torch.bfloat16) for w in self.W] if dtype == B.BF16 else self.W)
        # workspaces
        self.ws_layer = []
        bwd_bytes = 0
        for i, d in enumerate(self.desc):
            nbytes = max(B.conv_workspace_bytes(d, B.PASS_FORWARD),
                         B.conv_workspace_bytes(d, B.PASS_BACKWARD_WEIGHTS))
            self.ws_layer.append(torch.empty(nbytes, dtype=torch.uint8, device=device))
            if not (i == 0 and skip_first_dgrad):
                bwd_bytes = max(bwd_bytes, B.conv_workspace_bytes(d, B.PASS_BACKWARD_DATA))
        self.ws_bwd = torch.empty(max(bwd_bytes, 16), dtype=torch.uint8, device=device)
        # Repacked weights of the fused forward / data-gradient kernels, owned here and rewritten by ONE launch
        # whenever the weights change (set_parameters, sgd_step) instead of by every forward / backward call.
        self.packed_fwd, self.packed_bwd = [], []
        for i, d in enumerate(self.desc):
            nf = B.conv_packed_weights_bytes(d, B.PASS_FORWARD)
            nb = 0 if (i == 0 and skip_first_dgrad) else B.conv_packed_weights_bytes(d, B.PASS_BACKWARD_DATA)
            self.packed_fwd.append(torch.empty(nf, dtype=torch.uint8, device=device) if nf else None)
            self.packed_bwd.append(torch.empty(nb, dtype=torch.uint8, device=device) if nb else None)
        # activations
        self.X: List[Optional[torch.Tensor]] = [None] * len(self.layers)
        self.Y, self.P, self.A, self._dYd, self.dXl = [], [], [], [], []
        # dY of a layer whose model gradient multiplies the "rows" matrix [F][N * pitch]: written in that form by
        # the pooling / ReLU backward pass behind it (with the planes' sums for the bias gradient) and read as it
        # is by both backward passes of the convolution, instead of a dense tensor that the library would repack
        self.dYr, self.dYs, self.rows_ld = [], [], []
        self.Nrm, self.Sc, self.Dr, self.gN, self.gD = [], [], [], [], []   # normalised / scale / dropped; their gradients
        for i, (L, d) in enumerate(zip(self.layers, self.desc)):
            ho, wo = B.conv_output_dims(d)
            self.Y.append(torch.empty((L.N, L.F, ho, wo), dtype=self.tdtype, device=device))
            layout = B.conv_dy_rows_layout(self.desc_wgrad[i]) if (dy_rows and dtype == B.BF16) else None
            need_dx = not (i == 0 and skip_first_dgrad)
            if layout is not None and ((need_dx and self.packed_bwd[i] is None) or not (L.pool_after or L.relu)
                                       or (not L.pool_after and ho * wo > 2048)):
                layout = None
            self.rows_ld.append(layout[0] if layout else 0)
            self.dYr.append(torch.zeros((L.F, layout[0]), dtype=self.tdtype, device=device) if layout else None)
            self.dYs.append(torch.empty((L.F, L.N), dtype=torch.float32, device=device) if layout else None)
            self._dYd.append(None if layout else torch.empty((L.N, L.F, ho, wo), dtype=self.tdtype, device=device))
            if L.pool_after:
                po, pw = B.pool_output_dim(ho, 3, 2, ceil_mode), B.pool_output_dim(wo, 3, 2, ceil_mode)
                self.P.append(torch.empty((L.N, L.F, po, pw), dtype=self.tdtype, device=device))
                self.A.append(torch.empty((L.N, L.F, po, pw), dtype=torch.uint8, device=device))
            else:
                self.P.append(None)
                self.A.append(None)
            out = self.P[-1] if L.pool_after else self.Y[-1]
            self.Nrm.append(torch.empty_like(out) if L.lrn_after else None)
            self.Sc.append(torch.empty(out.shape, dtype=torch.float32, device=device) if L.lrn_after else None)
            self.gN.append(torch.empty_like(out) if L.lrn_after else None)
            self.Dr.append(torch.empty_like(out) if L.dropout_after > 0 else None)
            self.gD.append(torch.empty_like(out) if L.dropout_after > 0 else None)
            self.dXl.append(torch.empty((L.N, L.C, L.H, L.W), dtype=self.tdtype, device=device) if need_dx else None)
        # A convolution + ReLU layer directly in front of another rows-form layer: that layer's data gradient applies
        # the ReLU's mask and stores the result as this layer's rows matrix itself (with partial sums per column
        # tile instead of per plane), so neither a dense dX nor a separate ReLU backward pass exists for the pair.
        self.fused_front = [False] * len(self.layers)
        for i in range(len(self.layers) - 1):
            L = self.layers[i]
            if not (fuse_relu_dgrad and self.dYr[i] is not None and self.dYr[i + 1] is not None and L.relu
                    and not L.pool_after and not L.lrn_after and L.dropout_after == 0):
                continue
            per = B.conv_backward_data_relu_rows_sums(self.desc[i + 1])
            if per is None:
                continue
            self.fused_front[i] = True
            self.dYs[i] = torch.empty((L.F, per), dtype=torch.float32, device=device)
            self.dXl[i + 1] = None

    @property
    def dYc(self) -> List[torch.Tensor]:
        """Every layer's output gradient as a dense [N][F][Ho][Wo] tensor (a copy where the layer keeps the rows form)."""
        out = []
        for i, L in enumerate(self.layers):
            if self.dYr[i] is None:
                out.append(self._dYd[i])
                continue
            ho, wo = self.Y[i].shape[-2:]
            planes = self.dYr[i].view(L.F, L.N, -1)[:, :, :ho * wo]
            out.append(planes.permute(1, 0, 2).reshape(L.N, L.F, ho, wo).contiguous())
        return out

    # ------------------------------------------------------------------ parameters
    def set_parameters(self, Ws, bs) -> None:
        for i, (w, b) in enumerate(zip(Ws, bs)):
            self.W[i].copy_(torch.as_tensor(w, dtype=torch.float32))
            self.b[i].copy_(torch.as_tensor(b, dtype=torch.float32))
            if self.dtype == B.BF16:
                self.Wc[i].copy_(self.W[i])       # plumbing: the inputs are bf16-representable already
            self.VW[i].zero_()
            self.Vb[i].zero_()
        self.repack_weights()

    def repack_weights(self) -> None:
        """The fused kernels' copies of the current weights, all layers and both passes in launches of up to 16."""
        jobs = [(self.desc[i], B.PASS_FORWARD, self.Wc[i], p) for i, p in enumerate(self.packed_fwd) if p is not None]
        jobs += [(self.desc[i], B.PASS_BACKWARD_DATA, self.Wc[i], p) for i, p in enumerate(self.packed_bwd) if p is not None]
        for k in range(0, len(jobs), 16):
            d, ps, w, out = zip(*jobs[k:k + 16])
            B.conv_pack_weights(d, ps, w, out)

    def output_shape(self):
        last = self.P[-1] if self.P[-1] is not None else self.Y[-1]
        return tuple(last.shape)

    LRN = (5, 1e-4, 0.75, 1.0)   # channel window, alpha, beta, k of the network's normalisation layers

    # ------------------------------------------------------------------ passes
    def forward(self, X: torch.Tensor) -> torch.Tensor:
        cur = X
        for i, L in enumerate(self.layers):
            self.X[i] = cur
            if self.packed_fwd[i] is not None:
                B.conv_forward_packed(self.desc[i], cur, self.packed_fwd[i], self.b[i], self.Y[i], self.ws_layer[i])
            else:
                B.conv_forward(self.desc[i], cur, self.Wc[i], self.b[i], self.Y[i], self.ws_layer[i])
            cur = self.Y[i]
            if L.pool_after:
                B.maxpool_forward(cur, 3, 2, self.ceil_mode, self.P[i], self.A[i])
                cur = self.P[i]
            if L.lrn_after:
                B.lrn_forward(cur, *self.LRN, y=self.Nrm[i], scale=self.Sc[i])
                cur = self.Nrm[i]
            if L.dropout_after > 0:
                B.dropout_forward(cur, L.dropout_after, self.dropout_seed, i, y=self.Dr[i])
                cur = self.Dr[i]
        return cur

    def backward(self, dOut: torch.Tensor) -> Optional[torch.Tensor]:
        g = dOut
        for i in reversed(range(len(self.layers))):
            L, Y = self.layers[i], self.Y[i]
            if L.dropout_after > 0:
                B.dropout_backward(g, L.dropout_after, self.dropout_seed, i, dx=self.gD[i])
                g = self.gD[i]
            if L.lrn_after:
                B.lrn_backward(self.P[i] if L.pool_after else Y, g, self.Sc[i], *self.LRN, dx=self.gN[i])
                g = self.gN[i]
            rows = self.dYr[i]
            if self.fused_front[i]:
                pass                 # written by the data gradient of the layer behind
            elif rows is not None and L.pool_after:
                B.maxpool_backward_rows(g, self.A[i], self.P[i] if L.relu else None, Y.shape[-2], Y.shape[-1], 3, 2,
                                        self.ceil_mode, dx_rows=rows, plane_sums=self.dYs[i], ld=self.rows_ld[i])
            elif rows is not None:
                B.relu_backward_rows(Y, g, dx_rows=rows, plane_sums=self.dYs[i], ld=self.rows_ld[i])
            elif L.pool_after and L.relu:
                B.maxpool_relu_backward(g, self.A[i], self.P[i], Y.shape[-2], Y.shape[-1], 3, 2, self.ceil_mode,
                                        self._dYd[i])
            elif L.pool_after:
                B.maxpool_backward(g, self.A[i], Y.shape[-2], Y.shape[-1], 3, 2, self.ceil_mode, dx=self._dYd[i])
            elif L.relu:
                B.relu_backward(Y, g, self._dYd[i])
            else:
                self._dYd[i] = g     # no layer between the convolution and the incoming gradient

            def model_gradient():
                if rows is not None:
                    B.conv_backward_weights_rows(self.desc_wgrad[i], self.X[i], rows, self.dYs[i], self.dW[i], self.db[i],
                                                 self.ws_layer[i])
                else:
                    B.conv_backward_weights(self.desc_wgrad[i], self.X[i], self._dYd[i], self.dW[i], self.db[i],
                                            self.ws_layer[i])
            if self.side is not None:
                self.side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(self.side):
                    model_gradient()
            else:
                model_gradient()
            if i > 0 and self.fused_front[i - 1]:
                B.conv_backward_data_relu_rows(self.desc[i], rows, self.packed_bwd[i], self.Y[i - 1], dX_rows=self.dYr[i - 1],
                                               col_sums=self.dYs[i - 1], ld_out=self.rows_ld[i - 1], workspace=self.ws_bwd)
                g = None
                continue
            if self.dXl[i] is None:
                g = None
                break
            if rows is not None:
                B.conv_backward_data_rows(self.desc[i], rows, self.packed_bwd[i], self.dXl[i], self.ws_bwd)
            elif self.packed_bwd[i] is not None:
                B.conv_backward_data_packed(self.desc[i], self._dYd[i], self.packed_bwd[i], self.dXl[i], self.ws_bwd)
            else:
                B.conv_backward_data(self.desc[i], self._dYd[i], self.Wc[i], self.dXl[i], self.ws_bwd)
            g = self.dXl[i]
        if self.side is not None:
            torch.cuda.current_stream().wait_stream(self.side)
        return g

    def sgd_step(self, lr: float, momentum: float, weight_decay: float = 0.0) -> None:
        shadow = None
        if self.dtype == B.BF16:
            shadow = list(self.Wc) + [None] * len(self.b)
        B.sgd_momentum_step(self.W + self.b, self.VW + self.Vb, self.dW + self.db, lr, momentum,
                            weight_decay, shadow)
        self.repack_weights()

    def step(self, X: torch.Tensor, dOut: torch.Tensor, lr: float, momentum: float,
             weight_decay: float = 0.0) -> torch.Tensor:
        out = self.forward(X)
        self.backward(dOut)
        self.sgd_step(lr, momentum, weight_decay)
        return out

    # ------------------------------------------------------------------ state checks (plumbing, after a run)
    def tensor_health(self, W_start: Optional[Sequence[torch.Tensor]] = None) -> dict:
        """Finiteness and spread of the tensors the last step left: parameters, velocities, gradients, every
        layer's output and the last data gradient.  Reads tensors back with torch; no part of a step."""
        torch.cuda.synchronize()
        last_dx = next((d for d in self.dXl if d is not None), None)
        state = list(self.W) + list(self.b) + list(self.VW) + list(self.Vb) + list(self.dW) + list(self.db) + list(self.Y)
        if last_dx is not None:
            state.append(last_dx)
        h = {
            "finite": all(bool(torch.isfinite(t.float()).all()) for t in state),
            "zero_fraction_Y": [round(float((y == 0).float().mean()), 4) for y in self.Y],
            "max_abs_Y": [float(y.float().abs().max()) for y in self.Y],
            "max_abs_W": [float(w.abs().max()) for w in self.W],
            "std_W": [float(w.std()) for w in self.W],
            "max_abs_dW": [float(g.abs().max()) for g in self.dW],
        }
        if W_start is not None:
            h["max_abs_W_change"] = [float((w - w0).abs().max()) for w, w0 in zip(self.W, W_start)]
        if last_dx is not None:
            h["max_abs_dX_last"] = float(last_dx.float().abs().max())
            h["zero_fraction_dX_last"] = round(float((last_dx == 0).float().mean()), 4)
        return h

    @staticmethod
    def health_is_degenerate(h: dict, sigma: float = 0.01) -> bool:
        """True if a step ran on tensors that no longer look like the workload: something not finite, a layer
        whose ReLU output is (almost) all zero, vanished gradients, or weights that left N(0, sigma)."""
        return (not h["finite"] or any(z > 0.9 for z in h["zero_fraction_Y"]) or any(m == 0.0 for m in h["max_abs_dW"])
                or h.get("max_abs_dX_last", 1.0) == 0.0
                or any(not (0.5 * sigma < sd < 2.0 * sigma) for sd in h["std_W"]))
