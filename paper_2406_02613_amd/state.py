"""Block-interleaved storage of one shard's theta, m, v and gsum (acco_layout_t).

One buffer of shape (blocks, 4, block_elems): block b holds, one after the other, elements
[b*block_elems, (b+1)*block_elems) of theta, of m, of v and of gsum.  The four views
``theta, m, v, gsum`` (shape (blocks, block_elems), strides (4*block_elems, 1)) are what the
step entry points take; the binding derives the layout from their strides.  Allocation and
copies only - no arithmetic.
"""
from __future__ import annotations

DEFAULT_BLOCK_ELEMS = 8192      # 32 KiB per component: the fastest of 1 Ki .. 128 Ki elements on MI355X


class BlockedState:
    def __init__(self, n: int, block_elems: int = DEFAULT_BLOCK_ELEMS, device="cuda", alloc=None):
        """alloc(numel, dtype) -> zeroed flat tensor, for a caller that places the buffer itself."""
        import torch
        if block_elems < 4 or block_elems & (block_elems - 1):
            raise ValueError("block_elems must be a power of two >= 4")
        self.n, self.block = int(n), int(block_elems)
        self.blocks = (self.n + self.block - 1) // self.block
        if alloc is None:
            self.buf = torch.zeros(self.blocks, 4, self.block, dtype=torch.float32, device=device)
        else:
            self.buf = alloc(self.blocks * 4 * self.block, torch.float32).view(self.blocks, 4,
                                                                                 self.block)
        self.theta, self.m, self.v, self.gsum = (self.buf[:, c, :] for c in range(4))

    def load(self, name: str, planar) -> None:
        """Copy a planar fp32 tensor of n elements into component ``name``."""
        view = getattr(self, name)
        if planar.numel() != self.n:
            raise ValueError(f"expected {self.n} elements")
        full = self.n // self.block
        if full:
            view[:full].copy_(planar[:full * self.block].view(full, self.block))
        rem = self.n - full * self.block
        if rem:
            view[full, :rem].copy_(planar[full * self.block:])

    def planar(self, name: str):
        """A planar copy (n elements) of component ``name``."""
        return getattr(self, name).reshape(-1)[:self.n].clone()


DEFAULT_COMM_BLOCK_ELEMS = 16384  # 32 KiB of bf16 per worker and block: the fastest of 4 Ki .. 64 Ki


class InterleavedShards:
    """The W workers' bf16 communication buffers interleaved block by block in one buffer of
    shape (blocks, W, block_elems): ``shard(w)`` is the (blocks, block_elems) view of worker w
    with strides (W * block_elems, 1), which acco_accumulate_batch writes (out_layout) and the
    reduction entry points read (shard_layout); the binding derives the layout from the strides.
    Allocation only - no arithmetic."""

    def __init__(self, n: int, workers: int, block_elems: int = DEFAULT_COMM_BLOCK_ELEMS,
                 device="cuda", alloc=None):
        import torch
        if block_elems < 8 or block_elems & (block_elems - 1):
            raise ValueError("block_elems must be a power of two >= 8")
        self.n, self.W, self.block = int(n), int(workers), int(block_elems)
        self.blocks = (self.n + self.block - 1) // self.block
        if alloc is None:
            self.buf = torch.zeros(self.blocks, self.W, self.block, dtype=torch.bfloat16,
                                   device=device)
        else:
            self.buf = alloc(self.blocks * self.W * self.block, torch.bfloat16).view(
                self.blocks, self.W, self.block)
        self.shards = [self.buf[:, w, :] for w in range(self.W)]

    def shard(self, w: int):
        return self.shards[w]

    def planar(self, w: int):
        """A planar copy (n elements) of worker w's buffer."""
        return self.shards[w].reshape(-1)[:self.n].clone()
