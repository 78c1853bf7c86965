"""Paged expert weights: a page pool plus the page table that locates every
logical page of every expert in it (the paper's weight pages and page table,
appendix A.1).  Packing is done by the library's host packer."""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B


class PagedWeights:
    """Holds pages (uint8 [pool_pages, page_bytes]) and the page table (int32 [E, pages_per_expert]).

    ``order``: None puts logical pages in natural order; a permutation of
    range(pool_pages) (or a torch.Generator to draw one) scatters them, which
    must not change any result.  ``extra_pages`` adds unused slots to the pool.
    """

    def __init__(self, shape: B.MoEShape, W1, W3, W2, order=None, extra_pages: int = 0, pin: bool = False):
        self.shape = shape
        gu, d = B.pages_required(shape)
        self.pages_gu, self.pages_d, self.ppe = gu, d, gu + d
        n = shape.E * self.ppe
        self.pool_pages = n + int(extra_pages)
        if order is None:
            slots = torch.arange(n, dtype=torch.int32)
        elif isinstance(order, torch.Generator):
            slots = torch.randperm(self.pool_pages, generator=order)[:n].to(torch.int32)
        else:
            slots = torch.as_tensor(order, dtype=torch.int32)[:n]
        self.table_host = slots.reshape(shape.E, self.ppe).contiguous()
        self.pages_host = B.pack_weights(shape, W1, W3, W2, self.table_host, self.pool_pages, pin=pin)
        self.pages_dev: Optional[torch.Tensor] = None
        self.table_dev: Optional[torch.Tensor] = None

    def to_device(self, device="cuda", keep_host: bool = False) -> "PagedWeights":
        self.pages_dev = self.pages_host.to(device)
        self.table_dev = self.table_host.to(device)
        if not keep_host:
            self.pages_host = None
        return self

    def unpack(self):
        return B.unpack_weights(self.shape, self.pages_host, self.table_host)
