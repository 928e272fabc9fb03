"""Streams the per-layer chunk caches from pinned host memory into HBM beside the computation.

The chunk K/V store of Eq. 1 is far larger than one prompt needs and lives outside the GPU; a prompt only
needs, layer by layer, the blocks of its own chunks in their packed slots.  ``ChunkCacheStream`` keeps a small
ring of device buffers, fills buffer ``l % depth`` with layer ``l`` on a copy stream (a3_chunk_cache_load)
while earlier layers compute, and hands the buffers over with events.  Sequencing only.
"""
from __future__ import annotations

from typing import List, Sequence

import torch

from . import api


class ChunkCacheStream:
    """host_k[l][c], host_v[l][c]: pinned CPU tensors [chunk_len[c], Hkv, d] of layer l, chunk c
    (None for layers that use no cache).  ``depth`` device buffer pairs are cycled.
    With ``host_v`` None the blocks are 8-bit: host_k[l][c] is a pinned uint8 tensor of chunk_len[c] records of
    a3_q8_row_bytes (keys and values of the chunk's rows in one block); acquire() then hands out the device
    records for a3_rope_realign_q8."""

    def __init__(self, layout: api.Layout, shape, chunk_start, chunk_len, host_k: Sequence, host_v: Sequence = None,
                 depth: int = 2):
        assert depth >= 2
        self.layout, self.depth = layout, depth
        self.chunk_start, self.chunk_len = list(map(int, chunk_start)), list(map(int, chunk_len))
        self.host_k, self.host_v = host_k, host_v
        self.q8 = host_v is None
        T = layout.total_tokens
        if self.q8:
            row = api.a3_q8_row_bytes(layout)
            self.k = [torch.zeros((T, row), dtype=torch.uint8, device=layout.device) for _ in range(depth)]
            self.v = [None] * depth
        else:
            dt = api.torch_dtype(layout.dtype)
            mk = lambda: torch.zeros((T, shape.n_kv_heads, shape.head_dim), dtype=dt, device=layout.device)
            self.k = [mk() for _ in range(depth)]
            self.v = [mk() for _ in range(depth)]
        self.copy_stream = torch.cuda.Stream(device=layout.device)          # default priority
        self.loaded: List = [None] * depth       # event: buffer i holds its layer
        self.free: List = [None] * depth         # event: the consumer of buffer i is done with it

    def prefetch(self, l: int) -> None:
        """Enqueue layer l's copies on the copy stream (after the buffer's previous consumer has finished)."""
        if l >= len(self.host_k) or self.host_k[l] is None:
            return
        i = l % self.depth
        if self.free[i] is not None:
            self.copy_stream.wait_event(self.free[i])
        if self.q8:
            api.a3_chunk_cache_load_q8(self.layout, self.chunk_start, self.chunk_len, self.host_k[l], self.k[i],
                                       stream=self.copy_stream)
        else:
            api.a3_chunk_cache_load(self.layout, self.chunk_start, self.chunk_len, self.host_k[l], self.host_v[l],
                                    self.k[i], self.v[i], stream=self.copy_stream)
        ev = torch.cuda.Event()
        ev.record(self.copy_stream)
        self.loaded[i] = ev

    def acquire(self, l: int, stream=None):
        """(k_cat, v_cat) of layer l, or the layer's 8-bit records; the compute stream waits until the copies
        have landed."""
        i = l % self.depth
        (stream or torch.cuda.current_stream()).wait_event(self.loaded[i])
        return self.k[i] if self.q8 else (self.k[i], self.v[i])

    def release(self, l: int, stream=None) -> None:
        """The compute stream is done with layer l's buffers (recorded as an event)."""
        ev = torch.cuda.Event()
        ev.record(stream or torch.cuda.current_stream())
        self.free[l % self.depth] = ev


class ChunkFileStream:
    """The same hand-over as ChunkCacheStream for 8-bit chunk caches that live in FILES: one file per chunk holding
    the chunk's records layer after layer, layer l (>= first_layer) at byte offset
    (l - first_layer) * chunk_len[c] * a3_q8_row_bytes.  A worker thread reads layer l's blocks into a pinned
    staging buffer (a3_chunk_file_read, ``io_threads`` reader threads), enqueues the copies into device buffer
    l % depth on the copy stream (a3_chunk_cache_load_q8) and records the event the consumer waits for; staging
    buffer and device buffer are reused only after the copies, respectively the consumer, have passed them.
    Sequencing only; ``close()`` ends the worker and closes the files."""

    q8 = True

    def __init__(self, layout: api.Layout, shape, chunk_start, chunk_len, paths: Sequence[str], n_layers: int,
                 first_layer: int = 2, depth: int = 2, io_threads: int = 4):
        import concurrent.futures
        import os
        assert depth >= 2
        self.layout, self.depth, self.io_threads = layout, depth, io_threads
        self.chunk_start, self.chunk_len = list(map(int, chunk_start)), list(map(int, chunk_len))
        self.n_layers, self.first_layer = n_layers, first_layer
        self.row = api.a3_q8_row_bytes(layout)
        self.fds = [os.open(p, os.O_RDONLY) for p in paths]
        T = layout.total_tokens
        self.dev = [torch.zeros((T, self.row), dtype=torch.uint8, device=layout.device) for _ in range(depth)]
        total = sum(self.chunk_len) * self.row
        self.staging = [torch.empty(max(total, 1), dtype=torch.uint8).pin_memory() for _ in range(depth)]
        self.copy_stream = torch.cuda.Stream(device=layout.device)          # default priority
        self.copied: List = [None] * depth       # event: the copies out of staging buffer i have finished
        self.free: List = [None] * depth         # event: the consumer of device buffer i is done with it
        self.jobs = {}                           # layer -> future returning the "loaded" event
        self.pool = concurrent.futures.ThreadPoolExecutor(max_workers=1)

    def _load(self, l: int):
        i = l % self.depth
        if self.copied[i] is not None:
            self.copied[i].synchronize()         # staging buffer i is free again
        blocks, pos = [], 0
        for n in self.chunk_len:
            blocks.append(self.staging[i][pos:pos + n * self.row])
            pos += n * self.row
        offs = [(l - self.first_layer) * n * self.row for n in self.chunk_len]
        api.a3_chunk_file_read(self.fds, offs, [n * self.row for n in self.chunk_len], blocks, n_threads=self.io_threads)
        if self.free[i] is not None:
            self.copy_stream.wait_event(self.free[i])
        api.a3_chunk_cache_load_q8(self.layout, self.chunk_start, self.chunk_len, blocks, self.dev[i],
                                   stream=self.copy_stream)
        ev = torch.cuda.Event()
        ev.record(self.copy_stream)
        self.copied[i] = ev
        return ev

    def prefetch(self, l: int) -> None:
        """Hand layer l to the worker thread (after release() of the layer that used its buffer before)."""
        if l < self.first_layer or l >= self.n_layers or l in self.jobs:
            return
        self.jobs[l] = self.pool.submit(self._load, l)

    def acquire(self, l: int, stream=None):
        """The layer's device records; the compute stream waits until the copies have landed (and this thread
        until the file reads have: when storage is slower than the layers, this is where the time goes)."""
        ev = self.jobs.pop(l).result()
        (stream or torch.cuda.current_stream()).wait_event(ev)
        return self.dev[l % self.depth]

    def release(self, l: int, stream=None) -> None:
        ev = torch.cuda.Event()
        ev.record(stream or torch.cuda.current_stream())
        self.free[l % self.depth] = ev

    def close(self) -> None:
        import os
        self.pool.shutdown(wait=True)
        for fd in self.fds:
            os.close(fd)
        self.fds = []
