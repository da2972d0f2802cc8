"""Full-KV offload (Section 3.3): the full cache of every layer lives in pinned host memory,
only a few layers' K and V are on the device at a time, and the next layer is copied in while
the current one is verified.  The partial cache (a gathered copy of the kept blocks, see
specpv_gather_blocks) and the buffer stay on the device, so a partial step moves nothing over
PCIe; only a full verification / refresh walks the host copy.

Plumbing only (pinned memory, one copy stream, events): every step of the method still runs
in the HIP kernels behind the C ABI.
"""
import torch


class LayerPrefetcher:
    """Device staging slots for layers whose K / V live in pinned host memory.

    host_k, host_v: lists (one entry per layer) of pinned CPU tensors of one shape and dtype.
    Use per layer, in order:  prefetch(l + 1); k, v = acquire(l); ...kernels...; release(l).
    prefetch(l) may run at most `slots - 1` layers ahead of the layer being computed.
    """

    def __init__(self, host_k, host_v, device="cuda:0", slots=2):
        if len(host_k) != len(host_v) or not host_k:
            raise ValueError("host_k, host_v: one tensor per layer")
        for t in list(host_k) + list(host_v):
            if t.is_cuda or not t.is_pinned():
                raise ValueError("the offloaded cache must be pinned host memory (allocate it with pin_memory=True)")
            if t.shape != host_k[0].shape or t.dtype != host_k[0].dtype or not t.is_contiguous():
                raise ValueError("all layers: one shape, one dtype, contiguous")
        if slots < 2:
            raise ValueError("at least two slots (one computing, one arriving)")
        self.host_k, self.host_v = list(host_k), list(host_v)
        self.slots = slots
        self.device = torch.device(device)
        self.dev_k = [torch.empty(host_k[0].shape, dtype=host_k[0].dtype, device=self.device) for _ in range(slots)]
        self.dev_v = [torch.empty(host_k[0].shape, dtype=host_k[0].dtype, device=self.device) for _ in range(slots)]
        self.copy_stream = torch.cuda.Stream(device=self.device)          # default priority
        self.ready = [torch.cuda.Event() for _ in range(slots)]           # copy of the slot's tenant has landed
        self.free = [torch.cuda.Event() for _ in range(slots)]            # kernels of the previous tenant are done
        self.tenant = [None] * slots

    def prefetch(self, layer):
        """Starts the host-to-device copy of `layer` (asynchronous)."""
        slot = layer % self.slots
        if self.tenant[slot] == layer:
            return
        with torch.cuda.stream(self.copy_stream):
            self.copy_stream.wait_event(self.free[slot])      # no-op before the first release
            self.dev_k[slot].copy_(self.host_k[layer], non_blocking=True)
            self.dev_v[slot].copy_(self.host_v[layer], non_blocking=True)
            self.ready[slot].record(self.copy_stream)
        self.tenant[slot] = layer

    def acquire(self, layer):
        """K, V of `layer` on the device; the current stream waits for the copy."""
        slot = layer % self.slots
        if self.tenant[slot] != layer:
            self.prefetch(layer)
        torch.cuda.current_stream(self.device).wait_event(self.ready[slot])
        return self.dev_k[slot], self.dev_v[slot]

    def release(self, layer):
        """The kernels enqueued so far on the current stream were the last readers of `layer`."""
        slot = layer % self.slots
        self.free[slot].record(torch.cuda.current_stream(self.device))

    def write_back(self, layer, dim, lo, hi):
        """Copies rows [lo, hi) along `dim` (the token axis) of `layer` from its device slot back to
        the host copy, after the kernels enqueued so far (tokens committed by a full verification)."""
        slot = layer % self.slots
        if self.tenant[slot] != layer:
            raise ValueError("layer %d is not on the device" % layer)
        done = torch.cuda.Event()
        done.record(torch.cuda.current_stream(self.device))
        with torch.cuda.stream(self.copy_stream):
            self.copy_stream.wait_event(done)
            self.host_k[layer].narrow(dim, lo, hi - lo).copy_(self.dev_k[slot].narrow(dim, lo, hi - lo), non_blocking=True)
            self.host_v[layer].narrow(dim, lo, hi - lo).copy_(self.dev_v[slot].narrow(dim, lo, hi - lo), non_blocking=True)

    def synchronize(self):
        self.copy_stream.synchronize()
