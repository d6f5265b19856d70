"""Sequences libcnn calls into one training iteration of a layer list (paper Section 3.1 ordering:
forward through all layers, then per layer weight gradient BEFORE backpropagation, the first layer
skipping backpropagation, then one SGD update over the flat parameter arena).  With fuse_sgd the update
of a layer happens inside its weight gradient's reduction instead; that layer's backpropagation, which
needs the weights of this iteration, is then issued first.

This module only orders calls and owns buffers; all arithmetic happens inside libcnn kernels.
Every call's inputs and outputs stay alive in distinct buffers and are recorded in `self.trace`
so that tests can re-evaluate each call on exactly the tensors it consumed.
"""
import numpy as np
import torch

from . import binding as B
from . import synth


def carve_arrays(n_floats, count, dev):
    """`count` zeroed float arrays of n_floats each, cut from ONE device allocation, each start 16-byte aligned and
    shifted by a few KB against its neighbours.  The update that streams weights, gradients and momentum side by
    side ran at 6.8-6.9 TB/s on arrays laid out this way and at 6.3-6.4 TB/s on three separate allocations of the
    same sizes (same kernel, same launches), so every set of arrays that is walked in lock step is made here."""
    slot = (n_floats + 1023) // 1024 * 1024
    shift = [0, 5 * 1024, 11 * 1024, 19 * 1024]
    assert count <= len(shift)
    block = torch.zeros(slot * count + shift[count - 1], dtype=torch.float32, device=dev)
    return [block[i * slot + shift[i]: i * slot + shift[i] + n_floats] for i in range(count)]


class Net:
    def __init__(self, ctx, wl: synth.Workload, weights=None, record=False, fuse=True, fuse_pool=True, fuse_sgd=True,
                 resident_wt=True):
        """fuse=True folds every ReLU that follows a convolution into the convolution's store, and its derivative
        into the store of whatever produces the gradient in front of it (the next convolution's backpropagation or
        the max-pool backward); fuse=False calls one entry point per layer.
        fuse_pool (with fuse): a conv -> ReLU -> 2x2 max-pool chain becomes one call that stores only the pooled
        activation and the window positions, where the library serves the shape that way.
        fuse_sgd: step() lets each layer's weight-gradient reduction apply the SGD update (no stored gradient, no
        separate update pass), where the library serves the shape that way.
        resident_wt: every convolution that backpropagates keeps the mirrored transpose-weights (Section 2.3) beside its
        weights; backpropagation reads them, the folded update refreshes them, and they are re-made only after the
        weights were changed some other way."""
        self.ctx, self.wl, self.record, self.fuse = ctx, wl, record, fuse
        self.resident_wt = bool(resident_wt)
        self.fuse_sgd = bool(fuse_sgd)
        self.fuse_pool = bool(fuse and fuse_pool)
        self.layers = list(wl.layers)
        dev = torch.device("cuda")
        wshapes = synth.weight_shapes(wl)
        sizes = [int(np.prod(s)) for s in wshapes]
        # one contiguous arena per role so the SGD update is a single launch; each slice 16-byte aligned
        offs, total = [], 0
        for n in sizes:
            offs.append(total)
            total += (n + 3) // 4 * 4
        self.n_params = sum(sizes)
        self.arena_elems = total
        arenas = carve_arrays(total, 3 if wl.momentum != 0.0 else 2, dev)
        self.w_arena, self.dw_arena = arenas[0], arenas[1]
        self.v_arena = arenas[2] if wl.momentum != 0.0 else None
        self.w = [self.w_arena[o:o + n].view(s) for o, n, s in zip(offs, sizes, wshapes)]
        self.dw = [self.dw_arena[o:o + n].view(s) for o, n, s in zip(offs, sizes, wshapes)]
        self.v = ([self.v_arena[o:o + n].view(s) for o, n, s in zip(offs, sizes, wshapes)] if self.v_arena is not None
                  else [None] * len(sizes))
        if weights is not None:
            for dst, src in zip(self.w, weights):
                dst.copy_(torch.from_numpy(np.ascontiguousarray(src)))
        # activations: act[i] = output of layer i; act_in[i] = its input
        shp = synth.shapes(wl)
        self.x = torch.empty(wl.input_shape, dtype=torch.float32, device=dev)
        self.act, self.gact, self.arg = [], [], {}
        for i, (L, s) in enumerate(zip(self.layers, shp)):
            if L[0] == "flatten":
                # a view in both directions: the gradient written by the next layer lands in the
                # gradient buffer of the layer before
                self.act.append(None)
                self.gact.append(self.gact[i - 1].view(s))
            else:
                self.act.append(torch.empty(s, dtype=torch.float32, device=dev))
                self.gact.append(torch.empty(s, dtype=torch.float32, device=dev))
            if L[0] == "pool":
                self.arg[i] = torch.empty(s, dtype=torch.uint8, device=dev)
        self.gx = None  # gradient w.r.t. the network input is never needed (Section 3.1)
        n = wl.input_shape[0]
        self.labels = torch.zeros(n, dtype=torch.int32, device=dev)
        self.loss_per_sample = torch.empty(n, dtype=torch.float32, device=dev)
        self.trace = []
        self.wT = [None] * len(self.w)          # resident transpose-weights per convolution, made on first use
        self._wt_state = {}                     # weight index -> "fresh" | "stale" | "off" (not served)
        self._fc_fused = set()
        self._pooled_ok, self._pooled_first = None, False
        self.marks = None   # a list while a caller wants (op, layer, profile-entry count after the call) per call
        self._reserve()

    # ------------------------------------------------------------ workspace
    def _reserve(self):
        need = 0
        shp = [tuple(self.wl.input_shape)] + synth.shapes(self.wl)
        L_ = B.lib()
        for i, L in enumerate(self.layers):
            sin = shp[i]
            if L[0] == "conv":
                _, c, k, r, s, st, pad = L
                for op in (B.OP_CONV_FWD, B.OP_CONV_FWD_RELU_POOL, B.OP_CONV_BWD_DATA, B.OP_CONV_BWD_WEIGHT):
                    need = max(need, L_.cnn_workspace_bytes(op, sin[0], c, sin[2], sin[3], k, r, s, st, pad))
            elif L[0] == "fc":
                for op in (B.OP_FC_FWD, B.OP_FC_BWD):
                    need = max(need, L_.cnn_workspace_bytes(op, sin[0], L[1], 1, 1, L[2], 1, 1, 1, 0))
        self.ctx.reserve(need)

    def _rec(self, *item):
        if self.record:
            self.trace.append(item)
        if self.marks is not None:
            # bytes the call must move at least: every tensor it reads or writes once; the weights and velocity a
            # folded update rewrites in place count twice
            seen, nbytes = set(), 0
            for t in item[2:]:
                if isinstance(t, torch.Tensor) and t.data_ptr() not in seen:
                    seen.add(t.data_ptr())
                    nbytes += t.numel() * t.element_size()
            if "_sgd" in item[0]:
                wi = item[2]
                nbytes += sum(t.numel() * 4 for t in (self.w[wi], self.v[wi]) if t is not None)
            self.marks.append((item[0], item[1], self.ctx.profile_count(), nbytes))

    def _input_of(self, i):
        j = i - 1
        return self.x if j < 0 else self.act[j]

    # ------------------------------------------------------------ passes
    def _fused_relu_after(self, i):
        """conv at i whose ReLU (i+1) is folded into its store"""
        return (self.fuse and self.layers[i][0] == "conv" and i + 1 < len(self.layers)
                and self.layers[i + 1][0] == "relu")

    def forward(self):
        ctx, wi = self.ctx, 0
        skip = set()
        self._fc_fused = set()      # fully-connected layers whose activation was folded into their store
        for i, L in enumerate(self.layers):
            xin, kind = self._input_of(i), L[0]
            if i in skip:
                continue
            if kind == "conv":
                pooled = None
                if (self.fuse_pool and self._fused_relu_after(i) and i + 2 < len(self.layers)
                        and self.layers[i + 2][0] == "pool" and self.act[i].shape[2] % 2 == 0 and self.act[i].shape[3] % 2 == 0):
                    pooled = B.cnn_conv_fwd_relu_pool(ctx, xin, self.w[wi], L[5], L[6], out=self.act[i + 2],
                                                      arg_out=self.arg[i + 2])
                if pooled is not None:
                    self._rec("conv_fwd_relu_pool", i, wi, xin, self.w[wi], self.act[i + 2], self.arg[i + 2])
                    skip.update((i + 1, i + 2))
                elif self._fused_relu_after(i):
                    B.cnn_conv_fwd_relu(ctx, xin, self.w[wi], L[5], L[6], out=self.act[i + 1])
                    self._rec("conv_fwd_relu", i, wi, xin, self.w[wi], self.act[i + 1])
                    skip.add(i + 1)
                else:
                    B.cnn_conv_fwd(ctx, xin, self.w[wi], L[5], L[6], out=self.act[i])
                    self._rec("conv_fwd", i, wi, xin, self.w[wi], self.act[i])
                wi += 1
            elif kind == "fc":
                nxt = self.layers[i + 1][0] if i + 1 < len(self.layers) else None
                done = None
                if self.fuse and nxt in ("relu", "sigmoid"):
                    # the activation behind the layer goes into the GEMM's store; its input is never written
                    done = B.cnn_fc_fwd_act(ctx, xin, self.w[wi], nxt, out=self.act[i + 1])
                if done is not None:
                    self._rec("fc_fwd_act", i, wi, xin, self.w[wi], self.act[i + 1], nxt)
                    self._fc_fused.add(i)
                    skip.add(i + 1)
                else:
                    B.cnn_fc_fwd(ctx, xin, self.w[wi], out=self.act[i])
                    self._rec("fc_fwd", i, wi, xin, self.w[wi], self.act[i])
                wi += 1
            elif kind == "relu":
                B.cnn_relu_fwd(ctx, xin, out=self.act[i]); self._rec("relu_fwd", i, xin, self.act[i])
            elif kind == "sigmoid":
                B.cnn_sigmoid_fwd(ctx, xin, out=self.act[i]); self._rec("sigmoid_fwd", i, xin, self.act[i])
            elif kind == "pool":
                B.cnn_maxpool2_fwd(ctx, xin, out=self.act[i], arg_out=self.arg[i])
                self._rec("pool_fwd", i, xin, self.act[i], self.arg[i])
            elif kind == "flatten":
                self.act[i] = xin.view(xin.shape[0], -1)
        return self.act[-1]

    def loss(self):
        """Softmax cross-entropy on the last activation; fills the gradient of the last activation."""
        z = self.act[-1]
        B.cnn_softmax_xent(self.ctx, z, self.labels, loss_out=self.loss_per_sample, dz_out=self.gact[-1])
        self._rec("softmax_xent", len(self.layers) - 1, z, self.labels, self.loss_per_sample, self.gact[-1])
        return self.loss_per_sample

    def _pooled_wgrad_serves(self):
        """Can the first layer's weight gradient be taken from the gradient behind its ReLU + pool?"""
        if self._pooled_ok is None:
            L, n = self.layers[0], self.wl.input_shape
            self._pooled_ok = (L[0] == "conv" and self.fuse_pool and
                               B.conv_bwd_weight_unpool_serves(n[0], L[1], n[2], n[3], L[2], L[3], L[4], L[5], L[6]))
        return self._pooled_ok

    def _wt_for(self, wi):
        """The resident transpose-weights of convolution wi, current with its weights; None where not kept."""
        if not self.resident_wt or self._wt_state.get(wi) == "off":
            return None
        if self.wT[wi] is None:
            K, C, R, S = self.w[wi].shape
            self.wT[wi] = torch.empty((C, K, R, S), dtype=torch.float32, device=self.w[wi].device)
            self._wt_state[wi] = "stale"
        if self._wt_state[wi] == "stale":
            if B.cnn_conv_transpose_weights(self.ctx, self.w[wi], out=self.wT[wi]) is None:
                self._wt_state[wi], self.wT[wi] = "off", None
                return None
            self._wt_state[wi] = "fresh"
            if self.marks is not None:
                self.marks.append(("transpose_weights", -1, self.ctx.profile_count(), 0))
        return self.wT[wi]

    def _weights_changed(self, wi=None):
        for k in (range(len(self.w)) if wi is None else (wi,)):
            if self._wt_state.get(k) == "fresh":
                self._wt_state[k] = "stale"

    def _bwd_data(self, i, wi, dy, H, W, x_act=None, arg=None, out=None):
        """One of the three backpropagation forms of convolution i, from the resident transpose-weights where kept."""
        ctx, L = self.ctx, self.layers[i]
        wT = self._wt_for(wi)
        if wT is not None:
            r = B.cnn_conv_bwd_data_wt(ctx, dy, wT, H, W, L[5], L[6], x_act=x_act, arg=arg, out=out)
            if r is not None:
                return r
            self._wt_state[wi], self.wT[wi] = "off", None
        if arg is not None:
            return B.cnn_conv_bwd_data_unpool_relu(ctx, dy, self.w[wi], arg, x_act, L[5], L[6], out=out)
        if x_act is not None:
            return B.cnn_conv_bwd_data_relu(ctx, dy, self.w[wi], x_act, L[5], L[6], out=out)
        return B.cnn_conv_bwd_data(ctx, dy, self.w[wi], H, W, L[5], L[6], out=out)

    def _wgrad(self, i, wi, update):
        """Weight gradient of conv layer i; with update, applied to the weights on the spot."""
        ctx, L, xin, dy = self.ctx, self.layers[i], self._input_of(i), self.gact[i]
        if i == 0 and self._pooled_first:
            self._pooled_first = False
            dpool, arg = self.gact[2], self.arg[2]
            if update:
                B.cnn_conv_bwd_weight_unpool(ctx, xin, dpool, arg, L[3], L[4], L[5], L[6], w=self.w[wi], v=self.v[wi],
                                             lr=self.wl.lr, momentum=self.wl.momentum)
                self._rec("conv_bwd_weight_unpool_sgd", i, wi, xin, dpool, arg, self.w[wi], self.v[wi])
            else:
                B.cnn_conv_bwd_weight_unpool(ctx, xin, dpool, arg, L[3], L[4], L[5], L[6], out=self.dw[wi])
                self._rec("conv_bwd_weight_unpool", i, wi, xin, dpool, arg, self.dw[wi])
            return
        if update:
            done = None
            if self._wt_state.get(wi) == "fresh":       # the update keeps the resident transpose-weights current
                done = B.cnn_conv_bwd_weight_sgd_wt(ctx, xin, dy, self.w[wi], self.wT[wi], self.v[wi], L[5], L[6],
                                                    self.wl.lr, self.wl.momentum)
            if done is None:
                done = B.cnn_conv_bwd_weight_sgd(ctx, xin, dy, self.w[wi], self.v[wi], L[5], L[6], self.wl.lr, self.wl.momentum)
                if done is not None:
                    self._weights_changed(wi)
            if done is not None:
                self._rec("conv_bwd_weight_sgd", i, wi, xin, dy, self.w[wi], self.v[wi])
                return
        B.cnn_conv_bwd_weight(ctx, xin, dy, L[3], L[4], L[5], L[6], out=self.dw[wi])
        self._rec("conv_bwd_weight", i, wi, xin, dy, self.dw[wi])
        if update:
            self._sgd_layer(wi)

    def _sgd_layer(self, wi):
        self._weights_changed(wi)
        v = self.v[wi].view(-1) if self.v[wi] is not None else None
        B.cnn_sgd_update(self.ctx, self.w[wi].view(-1), self.dw[wi].view(-1), v, self.wl.lr, self.wl.momentum)
        if self.marks is not None:
            self.marks.append(("sgd_update", -1, self.ctx.profile_count(), 0))

    def backward(self, update=False):
        """Expects gact[-1] to hold the gradient of the last activation (from loss() or set_upstream()).
        update=True also applies the SGD step, layer by layer, inside the weight gradients."""
        ctx = self.ctx
        wi = len(self.w)
        skip = set()
        for i in range(len(self.layers) - 1, -1, -1):
            L, kind = self.layers[i], self.layers[i][0]
            xin, dy = self._input_of(i), self.gact[i]
            first = i == 0
            dxb = None if first else self.gact[i - 1]
            if kind == "conv" or kind == "fc":
                wi -= 1
            if i in skip:
                continue
            # is the input of layer i the output of a ReLU that was folded into the convolution before it?
            relu_in = (not first) and i >= 2 and self.layers[i - 1][0] == "relu" and self._fused_relu_after(i - 2)
            if kind == "conv":
                if not update:       # the paper's order: weight gradient first
                    self._wgrad(i, wi, False)
                # is the input of layer i the output of ReLU -> pool behind a convolution (all folded in the forward pass)?
                pool_in = (self.fuse_pool and i >= 3 and self.layers[i - 1][0] == "pool" and self.layers[i - 2][0] == "relu"
                           and self._fused_relu_after(i - 3))
                unpooled = None
                if pool_in and i == 3 and self._pooled_wgrad_serves():
                    # the convolution in front of that ReLU + pool is the first layer: only its weight gradient wants
                    # the gradient, and it takes it at pooled size (Section 3.1: no backpropagation there)
                    self._bwd_data(i, wi, dy, xin.shape[2], xin.shape[3], x_act=xin, out=self.gact[i - 1])
                    self._rec("conv_bwd_data_relu", i, wi, dy, self.w[wi], xin, self.gact[i - 1])
                    skip.update((i - 1, i - 2))
                    self._pooled_first = True
                elif not first and pool_in:
                    # gradient in front of that ReLU + pool, straight into the earlier convolution's slot
                    unpooled = self._bwd_data(i, wi, dy, xin.shape[2], xin.shape[3], x_act=xin, arg=self.arg[i - 1],
                                              out=self.gact[i - 3])
                if unpooled is not None:
                    self._rec("conv_bwd_data_unpool_relu", i, wi, dy, self.w[wi], self.arg[i - 1], xin, self.gact[i - 3])
                    skip.update((i - 1, i - 2))
                elif not first and not (pool_in and i == 3 and self._pooled_first):
                    if relu_in:      # gradient in front of that ReLU, straight into the earlier convolution's slot
                        self._bwd_data(i, wi, dy, xin.shape[2], xin.shape[3], x_act=xin, out=self.gact[i - 2])
                        self._rec("conv_bwd_data_relu", i, wi, dy, self.w[wi], xin, self.gact[i - 2])
                        skip.add(i - 1)
                    else:
                        self._bwd_data(i, wi, dy, xin.shape[2], xin.shape[3], out=dxb)
                        self._rec("conv_bwd_data", i, wi, dy, self.w[wi], dxb)
                if update:           # backpropagation has read this iteration's weights: they may change now
                    self._wgrad(i, wi, True)
            elif kind == "fc":
                dx_out = None if first else dxb.view(xin.shape)
                done = None
                # is the input of layer i the output of an activation that was folded into the fully-connected layer
                # before it?  Then its derivative goes into this layer's backpropagation store, and the gradient lands
                # in front of the activation
                act_in = self.layers[i - 1][0] if (i >= 2 and (i - 2) in self._fc_fused) else None
                if act_in is not None:
                    dz_out = self.gact[i - 2].view(xin.shape)
                    if update:
                        done = B.cnn_fc_bwd_sgd_act(ctx, xin, self.w[wi], dy, act_in, self.v[wi], dz_out=dz_out,
                                                    lr=self.wl.lr, momentum=self.wl.momentum)
                        if done is not None:
                            self._rec("fc_bwd_sgd_act", i, wi, xin, self.w[wi], dy, dz_out, self.v[wi], act_in)
                    if done is None:
                        done = B.cnn_fc_bwd_act(ctx, xin, self.w[wi], dy, act_in, dz_out=dz_out, dw_out=self.dw[wi])
                        if done is not None:
                            self._rec("fc_bwd_act", i, wi, xin, self.w[wi], dy, dz_out, self.dw[wi], act_in)
                            if update:
                                self._sgd_layer(wi)
                    if done is not None:
                        skip.add(i - 1)
                        continue
                if update:
                    done = B.cnn_fc_bwd_sgd(ctx, xin, self.w[wi], dy, self.v[wi], need_dx=not first, dx_out=dx_out,
                                            lr=self.wl.lr, momentum=self.wl.momentum)
                if done is not None:
                    self._rec("fc_bwd_sgd", i, wi, xin, self.w[wi], dy, dx_out, self.v[wi])
                else:
                    B.cnn_fc_bwd(ctx, xin, self.w[wi], dy, need_dx=not first, need_dw=True, dx_out=dx_out, dw_out=self.dw[wi])
                    self._rec("fc_bwd", i, wi, xin, self.w[wi], dy, dx_out, self.dw[wi])
                    if update:
                        self._sgd_layer(wi)
            elif kind == "relu":
                # with the forward ReLU folded into the convolution only its output exists; a > 0 <=> z > 0
                mask = self.act[i] if (i >= 1 and (self._fused_relu_after(i - 1) or (i - 1) in self._fc_fused)) else xin
                B.cnn_relu_bwd(ctx, mask, dy, out=dxb); self._rec("relu_bwd", i, mask, dy, dxb)
            elif kind == "sigmoid":
                B.cnn_sigmoid_bwd(ctx, self.act[i], dy, out=dxb); self._rec("sigmoid_bwd", i, self.act[i], dy, dxb)
            elif kind == "pool":
                if relu_in:
                    B.cnn_maxpool2_relu_bwd(ctx, dy, self.arg[i], self.act[i], xin.shape[2], xin.shape[3],
                                            out=self.gact[i - 2])
                    self._rec("pool_relu_bwd", i, dy, self.arg[i], self.act[i], self.gact[i - 2])
                    skip.add(i - 1)
                else:
                    B.cnn_maxpool2_bwd(ctx, dy, self.arg[i], xin.shape[2], xin.shape[3], out=dxb)
                    self._rec("pool_bwd", i, dy, self.arg[i], dxb)
            # flatten: nothing to do, gact[i] aliases gact[i-1]
        return None

    def sgd(self):
        self._weights_changed()
        B.cnn_sgd_update(self.ctx, self.w_arena, self.dw_arena, self.v_arena, self.wl.lr, self.wl.momentum)
        if self.marks is not None:
            self.marks.append(("sgd_update", -1, self.ctx.profile_count(), 0))

    # ------------------------------------------------------------ helpers
    def set_input(self, x_np, labels_np=None):
        self.x.copy_(torch.from_numpy(x_np))
        if labels_np is not None:
            self.labels.copy_(torch.from_numpy(labels_np))

    def set_upstream(self, g_np):
        self.gact[-1].copy_(torch.from_numpy(g_np))

    def step(self):
        """One full iteration of the workload: forward, (loss), backward, (SGD)."""
        self.trace.clear()
        self.forward()
        if self.wl.loss:
            self.loss()
        if self.wl.sgd and self.fuse_sgd:
            self.backward(update=True)
        else:
            self.backward()
            if self.wl.sgd:
                self.sgd()
