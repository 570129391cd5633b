"""The memory pot of Continual Context Distillation (paper Sec. 3.2) as a thin driver around ccd_compress.

A pot holds at most n_cap cached tokens per (layer, KV head).  New context is appended until the pot is
full; then the catalyst-prompt queries of that moment score the cache and ccd_compress keeps k entries per
head in place, after which appending continues behind them.  Novelty is carried per head, because after
the first distillation heads no longer hold the same tokens in the same slots (Sec. 3.3.1).

Only buffer bookkeeping happens here; appending, scoring, selection and compaction all run in the library's kernels
(the append stands in for the model forward that would write new keys and values).
"""
from __future__ import annotations

import torch

from . import infinipot as ip


class MemoryPot:
    def __init__(self, B, L, Hkv, d, n_cap, k, T, *, dtype=torch.bfloat16, pool_w=7, pool_mode=ip.CCD_POOL_MAX,
                 device="cuda"):
        self.B, self.L, self.Hkv, self.d, self.n_cap, self.k, self.T = B, L, Hkv, d, n_cap, k, T
        self.pool_w, self.pool_mode = pool_w, pool_mode
        self.K = torch.zeros((B, L, Hkv, n_cap, d), dtype=dtype, device=device)
        self.V = torch.zeros_like(self.K)
        self.novelty = torch.zeros((B, L, Hkv, n_cap), dtype=torch.float32, device=device)
        self.keep_idx = torch.empty((B, L, Hkv, k), dtype=torch.int32, device=device)
        self.n_valid = 0
        self.calls = 0
        self._ws = None

    @property
    def room(self) -> int:
        return self.n_cap - self.n_valid

    def append(self, K_new, V_new, novelty_new) -> None:
        """K_new, V_new [B, L, Hkv, m, d]; novelty_new [B, m] (one value per token, copied to every head)."""
        m = K_new.shape[3]
        assert m <= self.room, "pot overflow: distill first"
        shape = ip.make_shape(None, self.K, self.novelty, k=1, n_valid=self.n_valid)
        rc = ip.ccd_append(shape, self.K, self.V, self.novelty, K_new, V_new, novelty_new)
        assert rc == ip.CCD_OK, rc
        self.n_valid += m

    def distill(self, Q_cat, scores=None) -> int:
        """One CCD compression if the pot is full; returns the library's code (CCD_OK or CCD_NOOP)."""
        shape = ip.make_shape(Q_cat, self.K, self.novelty, k=self.k, T=self.T, pool_w=self.pool_w,
                              pool_mode=self.pool_mode, n_valid=self.n_valid)
        if self._ws is None:
            full = ip.make_shape(Q_cat, self.K, self.novelty, k=self.k, T=self.T, pool_w=self.pool_w,
                                 pool_mode=self.pool_mode, n_valid=self.n_cap)
            self._ws = ip.alloc_workspace(full)
        rc = ip.ccd_compress(shape, Q_cat, self.K, self.V, self.novelty, self.keep_idx, self._ws, scores=scores)
        if rc == ip.CCD_OK:
            self.n_valid = self.k
            self.calls += 1
        return rc
