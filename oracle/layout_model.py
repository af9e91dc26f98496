"""Pool layout model (test infrastructure only): where a cached token lives.

The paper fixes only that the cache is allocated in blocks (Section 2.2,
block-grained allocation) and that whole jobs' key-value tensors move between
GPU and host memory (Section 4.2).  The byte layout inside a block is this
build's choice, stated in the public header; this file writes that statement
out a second time, independently of the GPU code, in integer arithmetic, so
that append and bulk-write placement can be checked bit for bit.

Stated layout.  With e = bytes per element, x = 16 / e elements per 16-byte
vector, B tokens per block, H heads, D head_dim, a block holds 2*H*B*D
elements: first the K region, then the V region.

    K element (head h, slot s, dim d):  ((h * (D/x) + d // x) * B + s) * x + d % x
    V element (head h, slot s, dim d):  H*B*D + (h * B + s) * D + d

Logical token t of job j lives in block ``table[j][t // B]`` at slot ``t % B``.
"""
from __future__ import annotations

import numpy as np


class PoolLayout:
    def __init__(self, num_heads: int, head_dim: int, block_size: int, elem_bytes: int):
        assert 16 % elem_bytes == 0
        self.H, self.D, self.B, self.e = num_heads, head_dim, block_size, elem_bytes
        self.x = 16 // elem_bytes
        assert head_dim % self.x == 0
        self.block_elems = 2 * num_heads * block_size * head_dim
        self.block_bytes = self.block_elems * elem_bytes

    def k_offset(self, h, s, d):
        """Element offset inside a block of K[h][s][d] (numpy-broadcastable)."""
        h, s, d = np.asarray(h), np.asarray(s), np.asarray(d)
        return ((h * (self.D // self.x) + d // self.x) * self.B + s) * self.x + d % self.x

    def v_offset(self, h, s, d):
        h, s, d = np.asarray(h), np.asarray(s), np.asarray(d)
        return self.H * self.B * self.D + (h * self.B + s) * self.D + d

    def token_offsets(self):
        """(k_off, v_off): int64 [B][H][D] element offsets of every slot of a block."""
        s = np.arange(self.B, dtype=np.int64)[:, None, None]
        h = np.arange(self.H, dtype=np.int64)[None, :, None]
        d = np.arange(self.D, dtype=np.int64)[None, None, :]
        return self.k_offset(h, s, d), self.v_offset(h, s, d)

    def write_tokens(self, image: np.ndarray, table_row: np.ndarray, start: int,
                     K: np.ndarray, V: np.ndarray) -> None:
        """Place tokens K[i], V[i] ([n][H][D]) at logical positions start+i of one
        job into `image` ([num_blocks][block_elems], the pool's element dtype)."""
        n = K.shape[0]
        if n == 0:
            return
        k_off, v_off = self.token_offsets()
        pos = np.arange(start, start + n, dtype=np.int64)
        blocks = np.asarray(table_row, dtype=np.int64)[pos // self.B]
        if (blocks < 0).any() or (blocks >= image.shape[0]).any():
            raise ValueError("table row does not cover the written positions")
        slots = pos % self.B
        image[blocks[:, None, None], k_off[slots]] = K
        image[blocks[:, None, None], v_off[slots]] = V

    def read_tokens(self, image: np.ndarray, table_row: np.ndarray, start: int, n: int):
        k_off, v_off = self.token_offsets()
        pos = np.arange(start, start + n, dtype=np.int64)
        blocks = np.asarray(table_row, dtype=np.int64)[pos // self.B]
        slots = pos % self.B
        return image[blocks[:, None, None], k_off[slots]], image[blocks[:, None, None], v_off[slots]]


def kv_bytes_per_job(num_layers: int, hidden: int, s: int, t: int, elem_bytes: int = 2) -> int:
    """Bytes of one job's whole cache, all layers: K and V, `hidden` elements each
    per token per layer (paper Section 4.2: 4*l*h*(s+t) at two bytes per element)."""
    return 2 * elem_bytes * num_layers * hidden * (s + t)
