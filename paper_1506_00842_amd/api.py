"""Convenience layer over the C-ABI binding: allocates device buffers with
PyTorch and calls the entry points.  No arithmetic of the method happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import (ModelHandle, TUNER_ALGO_AUTO, TUNER_FP32, tuner_best_of, tuner_decode_range,
               tuner_mean_relative_error, tuner_predict_all, tuner_predict_indices,
               tuner_predict_topk, tuner_predict_topk_prepared, tuner_predict_all_prepared, tuner_prepare,
               tuner_sample_valid, tuner_sample_workspace_bytes,
               tuner_space_create, tuner_space_size, tuner_train_ensemble,
               tuner_train_workspace_bytes, tuner_workspace_bytes)


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
        self.prepared = False
        if self.k > 0:
            self.values = torch.empty(self.k, dtype=torch.float32, device=self.device)
            # uint32 payload kept in an int32 tensor (same bytes)
            self.indices = torch.empty(self.k, dtype=torch.int32, device=self.device)
            self.n_found = torch.zeros(1, dtype=torch.int32, device=self.device)

    def prepare(self, stream=None):
        """Packs tables and weights into the workspace once; topk() and predict_all() then use
        the prepared entry points until a call that repacks (predict_indices) is made."""
        tuner_prepare(self.space, self.model, self.workspace, stream)
        self.prepared = True

    def topk(self, begin: int = 0, count: int | None = None, merge: bool = False, stream=None):
        """Enqueues one call; results stay on the device (self.values, self.indices, self.n_found)."""
        count = self.n_configs - begin if count is None else count
        fn = tuner_predict_topk_prepared if self.prepared else tuner_predict_topk
        fn(self.space, self.model, begin, count, self.k, 1 if merge else 0,
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
        fn = tuner_predict_all_prepared if self.prepared else tuner_predict_all
        fn(self.space, self.model, begin, count, out, mask if want_mask else None, self.workspace, stream)
        return out, mask

    def decode(self, begin: int, count: int):
        digits = torch.empty((count, self.n_params), dtype=torch.int32, device=self.device)
        feats = torch.empty((count, self.n_params), dtype=torch.float32, device=self.device)
        valid = torch.empty(count, dtype=torch.uint8, device=self.device)
        tuner_decode_range(self.space, begin, count, digits, feats, valid)
        return digits, feats, valid

    def predict_indices(self, indices, want_mask: bool = True, stream=None):
        """indices: int32/uint32-bit tensor on the device -> (predictions f32[n], mask u8[n] or None)."""
        n = indices.numel()
        out = torch.empty(n, dtype=torch.float32, device=self.device)
        mask = torch.empty(n, dtype=torch.uint8, device=self.device) if want_mask else None
        tuner_predict_indices(self.space, self.model, n, indices, out, mask, self.workspace, stream)
        self.prepared = False          # the list evaluation packs the weights in its own layout
        return out, mask


def _as_index_tensor(indices, device):
    """uint32 configuration indices kept in an int32 tensor (same bytes)."""
    if isinstance(indices, torch.Tensor):
        return indices.to(device)
    a = np.ascontiguousarray(indices).astype(np.uint32).view(np.int32)
    return torch.from_numpy(a).to(device)


class Tuner:
    """The stages around the sweep for one space: sampling, training, metrics
    (device buffers from PyTorch; every computation in the library)."""

    def __init__(self, space, device: str = "cuda:0"):
        self.device = torch.device(device)
        self.space_desc = space
        self.space = tuner_space_create(space.radices, space.flat_values, space.scales,
                                        space.constraint_terms, space.constraint_bounds)
        self.n_params = len(space.radices)

    def sample_valid(self, seed: int, n_samples: int, max_draws: int, stream=None):
        """-> (indices int32-tensor[n_samples] holding uint32 bits, n_found int32[1]), on the device."""
        ws = torch.empty(tuner_sample_workspace_bytes(max_draws), dtype=torch.uint8, device=self.device)
        out = torch.empty(n_samples, dtype=torch.int32, device=self.device)
        found = torch.zeros(1, dtype=torch.int32, device=self.device)
        tuner_sample_valid(self.space, seed, n_samples, max_draws, out, found, ws, stream)
        self._keep = ws
        return out, found

    def train(self, n_members: int, hidden: int, indices, times, parts, initial_weights,
              epochs: int, learning_rate: float, momentum: float, want_loss: bool = True, stream=None,
              workgroups_per_network: int = 0, barrier_poll_limit: int = 0):
        """-> (weights f32[E * per], loss f32[E, epochs + 1] or None), on the device."""
        idx = _as_index_tensor(indices, self.device)
        n = idx.numel()
        t = torch.as_tensor(np.ascontiguousarray(times, dtype=np.float32)).to(self.device) \
            if not isinstance(times, torch.Tensor) else times.to(self.device)
        pt = torch.as_tensor(np.ascontiguousarray(parts, dtype=np.int32)).to(self.device) \
            if not isinstance(parts, torch.Tensor) else parts.to(self.device)
        w0 = torch.as_tensor(np.ascontiguousarray(initial_weights, dtype=np.float32)).to(self.device) \
            if not isinstance(initial_weights, torch.Tensor) else initial_weights.to(self.device)
        ws = torch.empty(tuner_train_workspace_bytes(self.space, n), dtype=torch.uint8, device=self.device)
        w = torch.empty_like(w0)
        loss = torch.zeros((n_members, epochs + 1), dtype=torch.float32, device=self.device) if want_loss else None
        tuner_train_ensemble(self.space, n_members, hidden, n, idx, t, pt, w0, epochs, learning_rate,
                             momentum, w, loss, ws, stream, workgroups_per_network, barrier_poll_limit)
        self._keep = (ws, idx, t, pt, w0)
        return w, loss

    def mean_relative_error(self, predictions, times, stream=None):
        m = torch.zeros(1, dtype=torch.float32, device=self.device)
        n = torch.zeros(1, dtype=torch.int32, device=self.device)
        tuner_mean_relative_error(predictions.numel(), predictions, times, m, n, stream)
        return m, n

    def best_of(self, times, stream=None):
        pos = torch.zeros(1, dtype=torch.int32, device=self.device)
        bt = torch.zeros(1, dtype=torch.float32, device=self.device)
        tuner_best_of(times.numel(), times, pos, bt, stream)
        return pos, bt


class _TrainedModel:
    """What Sweep needs of a model: n_members / widths / weights."""

    def __init__(self, n_members, widths, weights):
        self.n_members, self.widths, self.weights = n_members, list(widths), weights


def tune(space, measure, initial_weights, n_train: int, m: int, n_members: int = 11, hidden: int = 30,
         epochs: int = 1000, learning_rate: float = 0.125, momentum: float = 0.875, seed: int = 0,
         device: str = "cuda:0"):
    """The two-stage tuner of the paper's Section 5 around a caller-supplied measurement.

    measure(indices uint64[n]) -> float32[n] execution times (a value that is not a finite
    number > 0 marks a failed run); it stands for compiling and running the benchmark.
    Steps: n_train random valid configurations -> their times -> bagged ensemble (n_members
    networks P-hidden-1, network e trained without part e = every n_members-th sample) ->
    sweep of the whole space, the m lowest predictions -> their times -> the fastest.
    Every computation runs in the library; this function only moves the measurements in.
    Returns a dict (best_index, best_time, candidates, candidate_times, weights, final_loss).
    """
    tn = Tuner(space, device)
    idx_dev, found = tn.sample_valid(seed, n_train, min(1 << 24, 64 * n_train))
    n = int(found.item())
    if n == 0:
        raise ValueError("no valid configuration found")
    idx_dev = idx_dev[:n]
    idx = idx_dev.cpu().numpy().view(np.uint32).astype(np.uint64)
    times = np.ascontiguousarray(measure(idx), dtype=np.float32)
    parts = (np.arange(n) % n_members).astype(np.int32) if n_members > 1 else np.full(n, -1, np.int32)
    weights, loss = tn.train(n_members, hidden, idx_dev, times, parts, initial_weights, epochs,
                             learning_rate, momentum)
    model = _TrainedModel(n_members, [tn.n_params, hidden, 1], weights.cpu().numpy())
    sw = Sweep(space, model, m, device)
    sw.topk()
    _, cand = sw.topk_host()
    cand_times = np.ascontiguousarray(measure(cand), dtype=np.float32)
    pos, best_time = tn.best_of(torch.from_numpy(cand_times).to(tn.device))
    pos = int(pos.item())
    return {"best_index": int(cand[pos]) if pos >= 0 else None, "best_time": float(best_time.item()),
            "candidates": cand, "candidate_times": cand_times, "weights": model.weights,
            "final_loss": loss[:, -1].cpu().numpy()}
