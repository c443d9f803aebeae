"""Upload of a synthetic decode problem to GPU memory (plumbing for tests,
smoke and bench; no arithmetic of the method)."""
from __future__ import annotations

import numpy as np
import torch


class DeviceProblem:
    """Device tensors of one problem: the paged pool holds `num_pages` slots of
    which only the used ones are written."""

    def __init__(self, p, device="cuda:0", pool=None, poison_unused=False):
        """poison_unused: fill the whole pool with NaN before the used pages are
        written (pools of up to a million tokens only), so that a read of any other page shows."""
        dev = torch.device(device)
        self.p = p
        self.q_nope = p.q_nope.to(dev)
        self.q_rope = p.q_rope.to(dev)
        key = None
        if pool is None:
            state = torch.empty(p.num_pages, p.h_c, p.page_size, p.d_v, dtype=torch.bfloat16, device=dev)
            rope = torch.empty(p.num_pages, p.page_size, p.d_r, dtype=torch.bfloat16, device=dev)
            if p.key_pages is not None:
                key = torch.empty(p.num_pages, p.h_c, p.page_size, p.d_n, dtype=torch.bfloat16, device=dev)
            if poison_unused and p.num_pages * p.page_size <= 16384 * 64:
                state.fill_(float("nan"))
                rope.fill_(float("nan"))
                if key is not None:
                    key.fill_(float("nan"))
        else:
            state, rope = pool[:2]
            key = pool[2] if len(pool) > 2 else None
        n_used = len(p.page_ids)
        if n_used:
            ids = torch.from_numpy(np.asarray(p.page_ids, dtype=np.int64)).to(dev)
            step = 4096
            for i in range(0, n_used, step):      # bounded staging copies
                state[ids[i:i + step]] = p.state_pages[i:i + step].to(dev)
                rope[ids[i:i + step]] = p.rope_pages[i:i + step].to(dev)
                if key is not None:
                    key[ids[i:i + step]] = p.key_pages[i:i + step].to(dev)
        self.state_cache, self.rope_cache, self.key_cache = state, rope, key
        self.page_table = torch.from_numpy(p.table_pool).to(dev)
        self.seq_lens = torch.from_numpy(np.asarray(p.seq_lens, dtype=np.int32)).to(dev)

    def args(self):
        return (self.q_nope, self.q_rope, self.state_cache, self.rope_cache, self.page_table,
                self.seq_lens, self.p.scale)
