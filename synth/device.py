"""Input generation on the GPU for tables too large to draw on the host in reasonable time (the 14.9 GB
edge-feature table of the 20,000,000-event configuration).  Random draws and row access only."""
from __future__ import annotations

import numpy as np


def device_normal_table(n_rows: int, width: int, seed: int, chunk_rows: int = 1 << 20):
    """float32 [n_rows, width] ~ N(0, 1) drawn on cuda:0 with a seeded generator, in chunks."""
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    out = torch.empty(n_rows, width, dtype=torch.float32, device="cuda")
    for lo in range(0, n_rows, chunk_rows):
        out[lo:lo + chunk_rows].normal_(generator=gen)
    return out


class HostRowView:
    """What a host-side consumer needs of a device-resident table: its shape and rows by index
    (fetched on demand, returned as numpy)."""

    def __init__(self, table):
        self.table = table
        self.shape = tuple(table.shape)
        self.dtype = np.float32

    def __getitem__(self, idx):
        import torch
        idx = np.asarray(idx)
        flat = torch.from_numpy(np.ascontiguousarray(idx.reshape(-1), np.int64)).to(self.table.device)
        rows = self.table.index_select(0, flat).cpu().numpy()
        return rows.reshape(idx.shape + (self.shape[1],))

    def __len__(self):
        return self.shape[0]
