"""Placement of buffers by memory class (see acco_hbm_classify in include/acco.h).

On MI355X a kernel that reads two streams from different classes of the HBM at the same time
runs 8-10 % slower than with both in one class, and written streams do best in a class the
kernel does not read.  Virtual addresses do not show the class, so an ``HbmArena`` takes ONE
device allocation, has the library classify it by timing, and hands out tensors from the parts
that belong to a requested class.  Allocation and bookkeeping only - no arithmetic; the
classification itself runs in the C-ABI library.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

from . import binding as B

ALIGN = 1 << 21                      # hand-outs start on 2 MiB boundaries


class HbmArena:
    def __init__(self, nbytes: int, *, step_bytes: int = 1 << 30, probe_bytes: int = 512 << 20,
                 device="cuda", classes: Optional[Sequence[int]] = None):
        """nbytes of device memory, classified position by position (every step_bytes, probes of
        probe_bytes).  ``classes``: a ready classification instead (then nothing is allocated
        and `alloc` is not available - for planning and for tests of the bookkeeping)."""
        nbytes = int(nbytes) // ALIGN * ALIGN
        if nbytes < probe_bytes:
            raise ValueError("an arena must hold at least one probe")
        self.nbytes, self.step, self.probe = nbytes, int(step_bytes), int(probe_bytes)
        count = (nbytes - self.probe) // self.step + 1
        if classes is None:
            import torch
            self.torch = torch
            self.slab = torch.empty(nbytes, dtype=torch.uint8, device=device)
            scratch = torch.empty(self.probe, dtype=torch.uint8, device=device)
            self.classes, self.n_classes = B.acco_hbm_classify(self.slab, self.step, self.probe,
                                                               scratch)
            del scratch
        else:
            if len(classes) != count or min(classes) < 0:
                raise ValueError(f"expected {count} class numbers >= 0")
            self.torch, self.slab = None, None
            self.classes, self.n_classes = list(classes), max(classes) + 1
        # runs of positions of one class; the boundary between two runs lies somewhere between
        # the last position of the one and the end of the first probe of the other, so that
        # stretch is left unused
        self.runs: List[List[int]] = []          # [class, start, end, cursor]
        k = 0
        while k < count:
            j = k
            while j + 1 < count and self.classes[j + 1] == self.classes[k]:
                j += 1
            start = k * self.step + (self.probe // 2 if k > 0 else 0)
            end = j * self.step + self.probe // 2 if j + 1 < count else nbytes
            start = (start + ALIGN - 1) // ALIGN * ALIGN
            if end > start:
                self.runs.append([self.classes[k], start, end, start])
            k = j + 1

    def free_bytes(self) -> Dict[int, int]:
        out = {c: 0 for c in range(self.n_classes)}
        for c, _, end, cur in self.runs:
            out[c] += end - cur
        return out

    def largest_free(self) -> Dict[int, int]:
        """Per class, the largest single request it can still serve."""
        out = {c: 0 for c in range(self.n_classes)}
        for c, _, end, cur in self.runs:
            out[c] = max(out[c], end - cur)
        return out

    def take(self, nbytes: int, cls: int, spill: bool = True) -> Tuple[int, int]:
        """Reserve nbytes: (offset into the arena, class it lies in).  First fit in the runs of
        `cls`; with `spill`, else in the class with the most room left, and so on."""
        need = max(int(nbytes), 1)
        free = self.free_bytes()
        order = [cls] + ([c for c in sorted(free, key=lambda c: -free[c]) if c != cls]
                         if spill else [])
        for c in order:
            for run in self.runs:
                if run[0] == c and run[3] + need <= run[2]:
                    off = run[3]
                    run[3] = (off + need + ALIGN - 1) // ALIGN * ALIGN
                    return off, c
        raise MemoryError(f"arena: no room for {need} bytes (class {cls}, spill={spill}); "
                          f"largest free stretch per class: {self.largest_free()}")

    def alloc(self, numel: int, dtype, cls: int, *, spill: bool = True, zero: bool = False):
        """A contiguous tensor of `numel` elements of `dtype` inside class `cls`; if that class
        is full and `spill` is set, inside whichever class has room (the result's ``acco_class``
        attribute tells).  Nothing is ever given back: an arena lives as long as its buffers."""
        if self.slab is None:
            raise RuntimeError("this arena was built from a given classification: no memory")
        esz = self.torch.empty((), dtype=dtype).element_size()
        off, c = self.take(int(numel) * esz, cls, spill)
        t = self.slab[off:off + int(numel) * esz].view(dtype)
        if zero:
            t.zero_()
        t.acco_class = c
        return t

    def describe(self) -> str:
        gib = float(1 << 30)
        runs = ", ".join(f"class {c}: {s / gib:.1f}-{e / gib:.1f} GiB" for c, s, e, _ in self.runs)
        return f"{self.nbytes / gib:.1f} GiB in {self.n_classes} classes ({runs})"


def plan_roles(arena: Optional[HbmArena], needs: Dict[str, int]) -> Dict[str, int]:
    """Which class each role's buffers go to.  Roles (bytes needed in `needs`):
    ``owner``   what the owner's step kernels read together: theta, m, v, gsum and the W
                communication buffers;
    ``compute`` what the accumulation kernels read together: accumulators, stashes and the
                micro-batch gradients;
    ``out``     the bf16 parameter outputs, only written.
    The two reading roles get a class each, the bigger need the class with more room; the
    outputs go to a third class if there is one, else to the class the step kernels do not
    read."""
    if arena is None:
        return {}
    free = arena.free_bytes()
    by_room = sorted(free, key=lambda c: -free[c])
    readers = sorted(("owner", "compute"), key=lambda r: -needs.get(r, 0))
    plan = {readers[0]: by_room[0], readers[1]: by_room[1 % len(by_room)]}
    plan["out"] = by_room[2] if len(by_room) > 2 else plan["compute"]
    return plan
