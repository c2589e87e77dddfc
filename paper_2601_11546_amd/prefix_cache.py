"""Block-level prefix cache over the paged KV pool (Sec. 2.3 "Prefix Cache": the engine finds the longest cached
prefix of a prompt and skips its computation; the paper's engine keys whole KV blocks by a hash of their tokens).

A block is `page_size` consecutive tokens at a page-aligned position.  Its key chains the key of the block before it
with its own tokens, so a block matches only behind the same prefix.  Full prompt blocks are registered when a
request is admitted (they are written by the batch that admits it); later requests whose prompts begin with the same
blocks name the same pages in their block tables and compute only what follows.  Pages of finished requests that
carry a key stay cached until the pool needs them (least recently used first); pages without a key (a partial last
block, generated tokens) return to the free list at once.

Host-side bookkeeping only: page ids in, page ids out.  `ready` tells the caller whether a shared block was written by
an earlier batch (it may then be declared as part of a shared prefix to the library) or is being written by the
batch under construction (then it is shared through the block tables only).
"""
from __future__ import annotations

import hashlib
from collections import OrderedDict

import numpy as np


class BlockPrefixCache:
    def __init__(self, num_pages: int, page_size: int):
        self.P, self.num_pages = page_size, num_pages
        self.free = list(range(num_pages - 1, -1, -1))
        self.by_key = {}                         # block key -> page
        self.key_of = [None] * num_pages         # page -> block key or None
        self.refs = [0] * num_pages
        self.ready = [False] * num_pages
        self.idle = OrderedDict()                # keyed pages with no user, least recently used first
        self.hits = self.misses = 0              # tokens served from the cache / computed, over all acquisitions

    # ---- keys
    def block_keys(self, tokens: np.ndarray) -> list:
        """Chained keys of the full blocks of a token sequence."""
        keys, prev = [], b""
        t = np.ascontiguousarray(tokens, np.int32)
        for i in range(len(t) // self.P):
            prev = hashlib.blake2b(prev + t[i * self.P:(i + 1) * self.P].tobytes(), digest_size=16).digest()
            keys.append(prev)
        return keys

    def match(self, tokens: np.ndarray) -> int:
        """Leading tokens of the prompt the cache holds: whole blocks, and never the whole prompt (its last token is
        always computed, so that the request has a query row)."""
        n = 0
        for k in self.block_keys(tokens):
            if k not in self.by_key or (n + self.P) >= len(tokens):
                break
            n += self.P
        return n

    # ---- pages
    def _take(self) -> int:
        if self.free:
            return self.free.pop()
        if not self.idle:
            raise RuntimeError("KV page pool exhausted: every page is in use")
        page, _ = self.idle.popitem(last=False)              # evict the least recently used cached block
        del self.by_key[self.key_of[page]]
        self.key_of[page] = None
        self.ready[page] = False
        return page

    def pages_available(self) -> int:
        return len(self.free) + len(self.idle)

    def acquire(self, tokens: np.ndarray, extra_tokens: int):
        """Pages for a request with this prompt that will grow by extra_tokens.  Returns (pages, cached tokens,
        cached tokens whose blocks an earlier batch has written)."""
        P = self.P
        keys = self.block_keys(tokens)
        n_blocks = (len(tokens) + extra_tokens + P - 1) // P
        cached = self.match(tokens) // P
        if n_blocks - cached > self.pages_available() - sum(1 for k in keys[:cached] if self.by_key[k] in self.idle):
            raise RuntimeError("KV page pool exhausted: lower the scheduler's cap or enlarge the pool")
        pages, n_ready, all_ready = [], 0, True
        for i in range(cached):                               # shared blocks
            page = self.by_key[keys[i]]
            if self.refs[page] == 0:
                del self.idle[page]
            self.refs[page] += 1
            pages.append(page)
            all_ready = all_ready and self.ready[page]
            n_ready += P if all_ready else 0
        for i in range(cached, n_blocks):                     # blocks this request writes
            page = self._take()
            self.refs[page] = 1
            if i < len(keys) and keys[i] not in self.by_key:  # a full prompt block: later requests may share it
                self.by_key[keys[i]] = page
                self.key_of[page] = keys[i]
            pages.append(page)
        self.hits += cached * P
        self.misses += len(tokens) - cached * P
        return pages, cached * P, n_ready

    def acquire_private(self, n_pages: int) -> list:
        """Pages that take no part in sharing (no keys): for a computation that must not touch cached blocks."""
        if n_pages > self.pages_available():
            raise RuntimeError("KV page pool exhausted")
        pages = [self._take() for _ in range(n_pages)]
        for page in pages:
            self.refs[page] = 1
        return pages

    def mark_ready(self, pages) -> None:
        """The batch that wrote these pages has run."""
        for page in pages:
            if self.key_of[page] is not None:
                self.ready[page] = True

    def release(self, pages) -> None:
        for page in pages:
            self.refs[page] -= 1
            assert self.refs[page] >= 0
            if self.refs[page] == 0:
                if self.key_of[page] is None:
                    self.free.append(page)
                else:
                    self.idle[page] = None                    # most recently used end

    def check(self) -> None:
        """Bookkeeping invariants (used by the tests)."""
        used = sum(1 for r in self.refs if r > 0)
        assert used + len(self.free) + len(self.idle) == self.num_pages
        assert all(self.refs[p] == 0 and self.key_of[p] is not None for p in self.idle)
        assert all(self.refs[p] == 0 and self.key_of[p] is None for p in self.free)
        assert all(self.key_of[p] == k for k, p in self.by_key.items())
