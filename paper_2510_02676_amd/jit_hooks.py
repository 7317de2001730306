"""Just-in-time decode as PyTorch forward hooks (paper Section 3.3: compressed layers stay resident, a
layer's weights are decoded into a shared buffer right before its forward pass, and the buffer is handed
on to later layers).

A thin adapter over ``ecf8.Jit``: the pre-hook of layer l makes the current stream wait for the layer's
decode, points the layer's weight attributes at the decoded views and queues the decode of layer l + 1;
the post-hook releases the buffer.  All work is done by the library's calls; nothing here touches the bytes.
"""
import torch

from . import ecf8


class JitHooks:
    """layers: the modules in execution order.  names[l]: the attributes of layers[l] that receive the
    decoded tensors, in the order of the layer's tensors in `jit` (an ``ecf8.Jit`` over the same layers;
    it needs two buffers or more for the decode of layer l + 1 to overlap layer l).  The attributes are
    plain tensors of raw E4M3 bytes (uint8), or views of them as ``torch.float8_e4m3fn`` when
    `as_fp8` is set; outside a layer's forward pass they hold an empty tensor."""

    def __init__(self, layers, names, jit, as_fp8=False):
        if len(layers) != len(names):
            raise ValueError("one list of attribute names per layer")
        self.layers, self.names, self.jit, self.as_fp8 = list(layers), [list(n) for n in names], jit, as_fp8
        self.n_buffers = len(jit.buffers)
        self._handles = []
        self._empty = torch.empty(0, dtype=torch.uint8, device=jit.buffers[0].device)
        self._queued = set()
        for l, m in enumerate(self.layers):
            for n in self.names[l]:
                setattr(m, n, self._empty)
            self._handles.append(m.register_forward_pre_hook(self._pre(l)))
            self._handles.append(m.register_forward_hook(self._post(l)))

    def _prefetch(self, l):
        if l not in self._queued:
            self.jit.prefetch(l)
            self._queued.add(l)

    def _pre(self, l):
        def hook(module, args):
            self._prefetch(l)                                   # a no-op when the previous layer already queued it
            views = self.jit.acquire(l, torch.cuda.current_stream())
            for n, v in zip(self.names[l], views):
                setattr(module, n, v.view(torch.float8_e4m3fn) if self.as_fp8 else v)
            if self.n_buffers > 1 and l + 1 < len(self.layers):
                self._prefetch(l + 1)                           # overlaps this layer's forward pass
        return hook

    def _post(self, l):
        def hook(module, args, output):
            self.jit.release(l, torch.cuda.current_stream())
            self._queued.discard(l)
            for n in self.names[l]:
                setattr(module, n, self._empty)
        return hook

    def remove(self):
        for h in self._handles:
            h.remove()
        self._handles = []
