"""Module streaming: the weights and calibration input of the next module travel from pinned host memory to one
of two device staging sets on a side stream while the current module iterates on the one resident state.

Plumbing only (torch tensors, streams and events at default priority); every computation is the library's.
Device memory stays that of ONE module (state, plane cache, workspace) plus two staging sets, whatever the
number of modules: this is what keeps the footprint independent of the depth of the model.
"""
from __future__ import annotations

import torch

NAMES = ("W1hat", "W2hat", "X")


def pin(module_inputs: dict) -> dict:
    """Copy one module's inputs (W1hat, W2hat, X; any device) into freshly allocated pinned host tensors."""
    out = {}
    for n in NAMES:
        t = module_inputs[n]
        out[n] = torch.empty(t.shape, dtype=t.dtype, pin_memory=True).copy_(t)
    return out


class ModuleStreamer:
    """Double-buffered host -> device staging of same-shaped modules.

    host_modules: list of dicts of PINNED host tensors (see pin()).  Iterating yields (layer, staged) where
    `staged` is the device dict of that layer, valid until the next item is requested; the copy of layer
    l + 1 is enqueued on the side stream before layer l is handed out, and a staging set is only overwritten
    after the main stream has passed the point where its previous module was released.
    """

    def __init__(self, host_modules, device="cuda"):
        assert host_modules, "no modules"
        for m in host_modules:
            for n in NAMES:
                assert m[n].is_pinned(), "host tensors must be pinned (allocate them with pin_memory=True)"
                assert m[n].shape == host_modules[0][n].shape and m[n].dtype == host_modules[0][n].dtype
        self.host = host_modules
        self.device = torch.device(device)
        self.stage = [{n: torch.empty(host_modules[0][n].shape, dtype=host_modules[0][n].dtype, device=self.device)
                       for n in NAMES} for _ in range(2)]
        self.copy_stream = torch.cuda.Stream(device=self.device)     # default priority
        n = len(host_modules)
        self.copy_start = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        self.copied = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        self.freed = [torch.cuda.Event() for _ in range(n)]
        self.bytes_per_module = sum(host_modules[0][n].numel() * host_modules[0][n].element_size() for n in NAMES)

    @property
    def staging_bytes(self):
        return 2 * self.bytes_per_module

    def _enqueue_copy(self, layer):
        with torch.cuda.stream(self.copy_stream):
            if layer >= 2:
                self.copy_stream.wait_event(self.freed[layer - 2])   # the set's previous module is done
            self.copy_start[layer].record(self.copy_stream)
            for n in NAMES:
                self.stage[layer & 1][n].copy_(self.host[layer][n], non_blocking=True)
            self.copied[layer].record(self.copy_stream)

    def __iter__(self):
        main = torch.cuda.current_stream(self.device)
        n = len(self.host)
        self._enqueue_copy(0)
        for layer in range(n):
            if layer + 1 < n:
                self._enqueue_copy(layer + 1)
            main.wait_event(self.copied[layer])
            yield layer, self.stage[layer & 1]
            self.freed[layer].record(main)

    def copy_ms(self):
        """Per-module copy durations (call after a synchronize)."""
        return [self.copy_start[l].elapsed_time(self.copied[l]) for l in range(len(self.host))]
