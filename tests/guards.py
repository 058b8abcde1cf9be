"""Guard bands around device buffers: every buffer a test hands to the library sits between two
bands of a known byte pattern, which must be intact after the calls (an out-of-bounds store of a
tile kernel, before or behind a buffer, lands in one of them instead of in a neighbour)."""
import math

import torch

BAND = 4096       # bytes before and behind each buffer (keeps the 256-byte alignment the library asks for)
PATTERN = 0xA5


class Guards:
    def __init__(self, device="cuda"):
        self.device = device
        self.items = []

    def empty(self, shape, dtype, fill=None):
        """A tensor of `shape` / `dtype` whose storage has a band on either side."""
        shape = tuple(int(s) for s in (shape if hasattr(shape, "__len__") else (shape,)))
        nbytes = math.prod(shape) * torch.empty((), dtype=dtype).element_size()
        body = (nbytes + 255) // 256 * 256
        raw = torch.full((BAND + body + BAND,), PATTERN, dtype=torch.uint8, device=self.device)
        view = raw[BAND:BAND + nbytes].view(dtype).view(shape)
        if fill is not None:
            view.fill_(fill)
        self.items.append((raw, nbytes))
        return view

    def like(self, t):
        return self.empty(t.shape, t.dtype)

    def wrap_layer(self, layer):
        """Replace every buffer the layer owns by a guarded one of the same shape and type; returns self."""
        for name in layer._BUFFERS:
            t = getattr(layer, name, None)
            if t is not None:
                setattr(layer, name, self.like(t))
        return self

    def check(self):
        torch.cuda.synchronize()
        for i, (raw, nbytes) in enumerate(self.items):
            assert bool((raw[:BAND] == PATTERN).all()), "bytes before buffer %d were written" % i
            # the tail of the last 256-byte block behind the buffer's own bytes belongs to the band too
            assert bool((raw[BAND + nbytes:] == PATTERN).all()), "bytes behind buffer %d were written" % i
