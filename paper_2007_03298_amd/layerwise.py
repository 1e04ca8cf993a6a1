"""Layer-by-layer synchronisation on side streams (Sec. V-A1; Sec. IV-A).

The paper hooks into backpropagation: the backward hook of a layer applies the
worker's local update to that layer and starts the layer's group
synchronisation without blocking; the pre-forward hook of the layer waits for
that synchronisation before the next iteration uses the layer.  A model of L
layers is therefore synchronised with L calls per iteration (the ``L`` of the
``L*alpha`` latency term of Sec. IV-A), issued from the last layer to the first.

Here a layer is a column segment of the replica stacks and a synchronisation is
one ``ds_group_sync_opt`` launch on the segment's columns.  The launches go
round-robin to K side streams; a "fork" event makes the side streams start
after whatever the caller's stream has enqueued so far (the gradients), one
event per layer marks that layer's synchronisation, and the caller's stream
waits for a layer's event where the pre-forward hook would.

Only launches, streams and events: every step of the method runs in the
library's kernels.  torch supplies the stream and event objects.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import torch

from . import binding as ds


class LayerwiseSync:
    def __init__(self, segments: Sequence[Tuple[int, int]], n_streams: int, device=None):
        if n_streams < 1:
            raise ValueError("at least one side stream")
        self.segments: List[Tuple[int, int]] = [(int(o), int(n)) for o, n in segments]
        # all streams at the default priority
        self.side = [torch.cuda.Stream(device=device) for _ in range(n_streams)]
        self.layer_done = [torch.cuda.Event() for _ in self.segments]
        self.fork = torch.cuda.Event()

    def backward(self, X, G, g_dtype: int, ldx: int, ldg: int, W: int, perm, off, lr: float,
                 V=None, ldv: int = 0, momentum: float = 0.0, weight_decay: float = 0.0,
                 S=None, lds: int = 0, swa_factor: float = 0.0, stream: Optional[torch.cuda.Stream] = None) -> None:
        """What the backward hooks of one iteration enqueue: for every layer, from
        the last to the first, its local update fused with its group average, on
        the next side stream, followed by the layer's event.  Returns at once."""
        main = stream if stream is not None else torch.cuda.current_stream()
        self.fork.record(main)
        for st in self.side:
            st.wait_event(self.fork)
        g_bytes = 2 if g_dtype == ds.DS_BF16 else 4
        x0, g0 = X.data_ptr(), G.data_ptr()
        v0 = V.data_ptr() if V is not None else 0
        s0 = S.data_ptr() if S is not None else 0
        extended = V is not None or S is not None or weight_decay != 0.0
        for k, layer in enumerate(reversed(range(len(self.segments)))):
            o, n = self.segments[layer]
            st = self.side[k % len(self.side)]
            opt = None
            if extended:
                opt = ds.local_opt(v0 + 4 * o if v0 else None, ldv, momentum, weight_decay,
                                   s0 + 4 * o if s0 else None, lds, swa_factor)
            ds.ds_group_sync_opt(x0 + 4 * o, g0 + g_bytes * o, g_dtype, n, ldx, ldg, W, perm, off, lr, opt, st)
            self.layer_done[layer].record(st)

    def wait_layer(self, layer: int, stream: Optional[torch.cuda.Stream] = None) -> None:
        """The pre-forward hook of one layer: `stream` goes on only after that layer's synchronisation."""
        (stream if stream is not None else torch.cuda.current_stream()).wait_event(self.layer_done[layer])

    def wait_all(self, stream: Optional[torch.cuda.Stream] = None) -> None:
        """All pre-forward hooks, first layer to last (the order the next forward pass meets them)."""
        for layer in range(len(self.segments)):
            self.wait_layer(layer, stream)
