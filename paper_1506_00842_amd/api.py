"""Convenience layer over the C-ABI binding: allocates device buffers with
PyTorch and calls the entry points.  No arithmetic of the method happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import (ModelHandle, TUNER_ALGO_AUTO, TUNER_FP32, tuner_decode_range, tuner_predict_all,
               tuner_predict_topk, tuner_space_create, tuner_space_size, tuner_workspace_bytes)


class Sweep:
    """A space + an ensemble resident on one GPU.

    `space` needs radices / flat_values / scales / constraint_terms /
    constraint_bounds; `model` needs n_members / widths / weights (fp32 numpy).
    """

    def __init__(self, space, model, k: int = 0, device: str = "cuda:0",
                 precision: int = TUNER_FP32, algo: int = TUNER_ALGO_AUTO):
        self.device = torch.device(device)
        self.space = tuner_space_create(space.radices, space.flat_values, space.scales,
                                        space.constraint_terms, space.constraint_bounds)
        self.n_configs = tuner_space_size(self.space)
        self.n_params = len(space.radices)
        self.weights = torch.from_numpy(np.ascontiguousarray(model.weights, dtype=np.float32)).to(self.device)
        self.model = ModelHandle(model.n_members, model.widths, self.weights, precision, algo)
        self.k = int(k)
        nbytes = tuner_workspace_bytes(self.space, self.model, self.k)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        if self.k > 0:
            self.values = torch.empty(self.k, dtype=torch.float32, device=self.device)
            # uint32 payload kept in an int32 tensor (same bytes)
            self.indices = torch.empty(self.k, dtype=torch.int32, device=self.device)
            self.n_found = torch.zeros(1, dtype=torch.int32, device=self.device)

    def topk(self, begin: int = 0, count: int | None = None, merge: bool = False, stream=None):
        """Enqueues one call; results stay on the device (self.values, self.indices, self.n_found)."""
        count = self.n_configs - begin if count is None else count
        tuner_predict_topk(self.space, self.model, begin, count, self.k, 1 if merge else 0,
                           self.values, self.indices, self.n_found, self.workspace, stream)

    def topk_host(self):
        """Copies the current result to the host: (values f32[n], indices u64[n])."""
        n = int(self.n_found.item())
        vals = self.values[:n].cpu().numpy()
        idx = self.indices[:n].cpu().numpy().view(np.uint32).astype(np.uint64)
        return vals, idx

    def predict_all(self, begin: int = 0, count: int | None = None, want_mask: bool = True,
                    out=None, mask=None, stream=None):
        count = self.n_configs - begin if count is None else count
        if out is None:
            out = torch.empty(count, dtype=torch.float32, device=self.device)
        if want_mask and mask is None:
            mask = torch.empty(count, dtype=torch.uint8, device=self.device)
        tuner_predict_all(self.space, self.model, begin, count, out, mask if want_mask else None,
                          self.workspace, stream)
        return out, mask

    def decode(self, begin: int, count: int):
        digits = torch.empty((count, self.n_params), dtype=torch.int32, device=self.device)
        feats = torch.empty((count, self.n_params), dtype=torch.float32, device=self.device)
        valid = torch.empty(count, dtype=torch.uint8, device=self.device)
        tuner_decode_range(self.space, begin, count, digits, feats, valid)
        return digits, feats, valid
