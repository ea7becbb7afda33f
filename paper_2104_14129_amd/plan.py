"""A whole network's saved activations handled as a few multi-tensor launches.

A training step saves dozens of activations of very different sizes (ResNet-50: 53 conv inputs,
26-822 MB each at batch 256).  `TensorSetPlan` groups the tensors of one step into size classes
(a multi-tensor launch is sized for its largest tensor, so a call should hold tensors of similar
size), builds the descriptor tables of `actq_*_multi` once, and then runs each stage of the path
(Sec. 4.1 statistics, Sec. 4.3 allocation over all (tensor, sample) items, Sec. 4.1/5.1
quantize + pack, unpack + dequantize) as one C-ABI call per class with pointers worked out
beforehand, so that the host stays ahead of launches that take 30-600 us.

Only argument marshalling happens here: every step of the path runs in the library's kernels.
"""
from __future__ import annotations

import ctypes

from . import binding as B


def size_classes(Ds, max_per_call: int = B.MAX_TENSORS_PER_CALL, small: int = 0):
    """Tensor indices grouped by element count, largest first.  A size that occurs once, or a
    class whose element counts add up to less than `small`, joins the next larger class (a launch
    is sized for its largest tensor and the surplus blocks of smaller ones exit at once, which is
    cheaper than a launch of its own that cannot fill the chip); no class exceeds `max_per_call`."""
    by_size = {}
    for l, D in enumerate(Ds):
        by_size.setdefault(int(D), []).append(l)
    classes = []
    for D in sorted(by_size, reverse=True):
        members = by_size[D]
        joins = len(members) == 1 or D * len(members) < small
        if classes and joins and len(classes[-1]) + len(members) <= max_per_call:
            classes[-1] = classes[-1] + members
            continue
        for i in range(0, len(members), max_per_call):
            classes.append(members[i:i + max_per_call])
    return classes


class TensorSetPlan:
    """Buffers, tables and launches for tensors x[l] of shape [N, Ds[l]] (one dtype, full groups).

    All items (tensor l, sample n) share one bit stream `packed`; item l*N + n has its width in
    `bits` and its byte offset in `offsets`, both written by the device-side allocator
    (`allocate`) or supplied by the caller (`set_widths`).  Tensor i of class k draws its noise
    with tag `tag_stride * k + i` (the multi-tensor call adds the position inside the call).
    """

    def __init__(self, xs, N: int, packed_capacity: int, noise_bits: int = 16, hf: int = B.ACTQ_HDR_F32,
                 seed: int = 15, G: int = B.G_DEFAULT, tag_stride: int = 1000, with_outputs: bool = True,
                 small_class_bytes: int = 200 << 20):
        import torch
        self.torch = torch
        self.xs = list(xs)
        self.N, self.G, self.hf, self.seed, self.noise_bits = int(N), int(G), int(hf), int(seed), int(noise_bits)
        self.Ds = [int(x.numel() // N) for x in self.xs]
        if any(D % G for D in self.Ds):
            raise ValueError("every tensor must consist of full groups")
        dev = self.xs[0].device
        self.dtype = self.xs[0].dtype
        self.dt = B.ACTQ_F16 if self.dtype == torch.float16 else B.ACTQ_F32
        L = len(self.xs)
        self.bits = torch.empty(N * L, dtype=torch.uint8, device=dev)
        self.offsets = torch.empty(N * L, dtype=torch.int64, device=dev)
        self.result = torch.zeros(2, dtype=torch.int64, device=dev)
        self.packed = torch.empty(int(packed_capacity), dtype=torch.uint8, device=dev)
        hdr_dtype = torch.int16 if hf == B.ACTQ_HDR_BF16 else torch.float32
        self.gmin = [torch.empty(N * (D // G), dtype=torch.float32, device=dev) for D in self.Ds]
        self.grange = [torch.empty(N * (D // G), dtype=torch.float32, device=dev) for D in self.Ds]
        self.header = [torch.empty(N * (D // G) * 2, dtype=hdr_dtype, device=dev) for D in self.Ds]
        self.outs = [torch.empty((N, D), dtype=self.dtype, device=dev) for D in self.Ds] if with_outputs else None
        # a class below ~200 MB cannot keep the chip busy for longer than a launch takes to start and drain
        self.classes = size_classes(self.Ds, small=small_class_bytes // (N * self.xs[0].element_size()))
        self.tags = {}
        self._tables, self._tag0 = [], []
        for k, members in enumerate(self.classes):
            entries = []
            for i, l in enumerate(members):
                e = {"x": self.xs[l], "gmin": self.gmin[l], "grange": self.grange[l], "header": self.header[l],
                     "bits": self.bits[l * N:(l + 1) * N], "offsets": self.offsets[l * N:(l + 1) * N], "D": self.Ds[l]}
                if with_outputs:
                    e["out"] = self.outs[l]
                entries.append(e)
                self.tags[l] = tag_stride * k + i
            self._tables.append(B.tensor_table(entries))
            self._tag0.append(tag_stride * k)
        self._tptr = [ctypes.addressof(t) for t in self._tables]
        self._tlen = [len(t) for t in self._tables]
        self._lib = B.lib()

    # ---- widths

    def allocate(self, w_dev, D_items_dev, budget_bits: int, widths: int = B.ACTQ_WIDTHS_POW2, stream=None):
        """Device-side greedy allocation over all N * L items (asynchronous; `result` = bytes, status)."""
        B.allocate_bits_device(w_dev, D_items_dev, budget_bits, widths, self.bits, self.offsets, self.result, self.G,
                               stream=stream)

    def set_widths(self, bits_host, offsets_host):
        torch = self.torch
        self.bits.copy_(torch.from_numpy(bits_host))
        self.offsets.copy_(torch.from_numpy(offsets_host))

    # ---- the three stages, one call per class; `between(k)` runs after class k's launch (event records)

    def _run(self, call, stream, between):
        sp = B._stream(stream)
        rc = 0
        for k in range(len(self.classes)):
            rc |= call(k, sp)
            if between is not None:
                between(k)
        if rc:
            raise B.ActqError(rc, B.last_error())

    def group_stats(self, stream=None, between=None):
        lib, N, G, dt = self._lib, self.N, self.G, self.dt
        self._run(lambda k, sp: lib.actq_group_stats_multi(self._tptr[k], self._tlen[k], dt, N, G, sp), stream, between)

    def quantize_pack(self, stream=None, between=None):
        lib, N, G, dt = self._lib, self.N, self.G, self.dt
        pk, cap = self.packed.data_ptr(), self.packed.numel()
        self._run(lambda k, sp: lib.actq_quantize_pack_multi(self._tptr[k], self._tlen[k], dt, N, G, self.seed,
                                                             self._tag0[k], self.noise_bits, pk, cap, self.hf, sp),
                  stream, between)

    def unpack_dequantize(self, stream=None, between=None):
        if self.outs is None:
            raise ValueError("plan was built without output tensors")
        lib, N, G, dt = self._lib, self.N, self.G, self.dt
        pk, cap = self.packed.data_ptr(), self.packed.numel()
        self._run(lambda k, sp: lib.actq_unpack_dequantize_multi(self._tptr[k], self._tlen[k], pk, cap, self.hf, N, G,
                                                                 dt, sp), stream, between)
