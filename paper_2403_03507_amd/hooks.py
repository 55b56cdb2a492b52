"""Per-layer weight updates during back-propagation (Sec. 4.3 of arXiv 2403.03507).

`PerLayerGaLore` registers a post-accumulate-grad hook on every GaLore matrix.  When the last
gradient of a layer has been accumulated, the hook calls `galore_step` for that layer's slice of
the tensor list and drops the gradients, so full-size gradients of at most one layer are alive at
a time and the optimizer work of layer l overlaps with the backward pass of layer l - 1.

Only marshalling lives here: every arithmetic step runs in the library.  The library's streams are
joined into torch's current stream by `finish()`, which the training loop calls after `backward()`
(before the next forward pass reads the weights).
"""
import torch

from . import binding as gb


class PerLayerGaLore:
    def __init__(self, layers, rank, lr, overlap_calls=True, **kwargs):
        """layers: list of lists of 2-D parameters (one inner list per transformer block, in the order
        the library should see them).  overlap_calls: False, True (two calls in flight) or 3 (three; pass
        workspace_factor=3 too, so that refreshes overlap as well).  kwargs go to `binding.GaLore`
        (update_gap, scale, moments, workspace_factor, ...)."""
        self.layers = [list(l) for l in layers]
        self.flat = [p for l in self.layers for p in l]
        for p in self.flat:
            assert p.dim() == 2 and p.is_cuda and p.is_contiguous(), "GaLore matrices must be contiguous 2-D CUDA parameters"
        self.first = []
        pos = 0
        for l in self.layers:
            self.first.append(pos)
            pos += len(l)
        self.lr = lr
        self.opt = gb.GaLore([p.data for p in self.flat], rank, **kwargs)
        self.opt.set_call_overlap(overlap_calls)
        # with overlapped calls the library reads a gradient on its own streams after the hook has
        # returned: the caching allocator is told so before the gradient is dropped
        self._lib_streams = self.opt.library_streams() if overlap_calls else []
        # the weights stay where they are: their argument arrays are marshalled once
        self._w_arrays = [gb.tensor_array(gb.desc(p.data) for p in l) for l in self.layers]
        self._ready = [0] * len(self.layers)
        self._handles = []
        for li, l in enumerate(self.layers):
            for p in l:
                self._handles.append(p.register_post_accumulate_grad_hook(self._make_hook(li)))

    def _make_hook(self, li):
        def hook(param):
            self._ready[li] += 1
            if self._ready[li] == len(self.layers[li]):
                self._ready[li] = 0
                self._step_layer(li)
        return hook

    def _step_layer(self, li):
        params = self.layers[li]
        grads = [p.grad for p in params]
        for p, g in zip(params, grads):
            assert g is not None and g.dtype == p.dtype and g.is_contiguous()
        gb.galore_step(self.opt.ctx, self._w_arrays[li], [gb.desc(g) for g in grads], self.first[li], len(params), self.lr)
        for g in grads:
            for st in self._lib_streams:
                g.record_stream(st)
        for p in params:
            p.grad = None

    def finish(self):
        """Call after backward(): orders the library's streams before torch's current stream."""
        self.opt.join()

    def close(self):
        for h in self._handles:
            h.remove()
        self._handles = []
        self.opt.close()
