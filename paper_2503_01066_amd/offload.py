"""Host offload of saved records and their prefetch during the backward walk (host orchestration only:
copies, streams and events; no arithmetic).

Section 4.3 of the paper: the activations a serving step leaves behind may not fit next to the serving
state, so they are copied to pinned host memory on a stream of their own and brought back when the trainer
needs them; Section 4.3.2: the backward pass consumes them one layer at a time, from the output layer to the
input layer, so the copy of layer l-1 can run while layer l computes.

`RecordStore` keeps one pinned host copy per layer and two device staging slots.  `offload(l, record)`
enqueues the device-to-host copies of layer l behind the work already on the caller's stream.
`prefetching_backward(...)` runs `alch_stack_backward` (or its adapter variant) with every layer's record
pointers aimed at the staging slot l % 2 and a `layer_ready` hook that (1) makes the compute stream wait
for layer l's host-to-device copy and (2) lets the copy of layer l-1 start as soon as the kernels of layer
l+1 -- the previous user of that slot -- have finished.
"""
import torch

from . import binding as B

KEYS = B.RECORD_KEYS + ("LSE",)


class RecordStore:
    def __init__(self, n_layers, example_record, keys=KEYS):
        """example_record: dict of device tensors with the shapes and dtypes of one layer's record."""
        self.keys = tuple(k for k in keys if example_record.get(k) is not None)
        self.n_layers = n_layers
        self.host = [{k: torch.empty(example_record[k].shape, dtype=example_record[k].dtype, pin_memory=True)
                      for k in self.keys} for _ in range(n_layers)]
        self.slots = [{k: torch.empty_like(example_record[k]) for k in self.keys} for _ in range(2)]
        self.copy_stream = torch.cuda.Stream()
        self.bytes_per_layer = sum(t.numel() * t.element_size() for t in self.host[0].values())

    def offload(self, layer, record, stream=None):
        """Device -> pinned host, asynchronous, ordered after what `stream` holds now."""
        stream = stream or torch.cuda.current_stream()
        done = torch.cuda.Event()
        done.record(stream)
        self.copy_stream.wait_event(done)
        with torch.cuda.stream(self.copy_stream):
            for k in self.keys:
                self.host[layer][k].copy_(record[k], non_blocking=True)
                record[k].record_stream(self.copy_stream)

    def _fetch(self, layer):
        """Pinned host -> staging slot layer % 2 on the copy stream; returns the event of its completion."""
        with torch.cuda.stream(self.copy_stream):
            for k in self.keys:
                self.slots[layer % 2][k].copy_(self.host[layer][k], non_blocking=True)
            ev = torch.cuda.Event()
            ev.record(self.copy_stream)
        return ev

    def prefetching_backward(self, backward, stream=None):
        """backward(saved_layers, hooks) must call alch_stack_backward[_lora] with those two arguments on `stream`.
        Returns what it returns."""
        stream = stream or torch.cuda.current_stream()
        L = self.n_layers
        ready = {}
        # the walk starts at layer L-1: its record and the next one go out first
        self.copy_stream.wait_stream(stream)
        for l in (L - 1, L - 2):
            if l >= 0:
                ready[l] = self._fetch(l)

        def layer_ready(_user, l):
            # kernels of layer l+1 are enqueued: once they are done its slot may be overwritten by layer l-1
            if l + 1 < L and l - 1 >= 0:
                freed = torch.cuda.Event()
                freed.record(stream)
                self.copy_stream.wait_event(freed)
                ready[l - 1] = self._fetch(l - 1)
            stream.wait_event(ready[l])
            return 0

        saved = [self.slots[l % 2] for l in range(L)]
        out = backward(saved, (layer_ready, None))
        # the staging slots must outlive the kernels that read them
        self.copy_stream.wait_stream(stream)
        return out
