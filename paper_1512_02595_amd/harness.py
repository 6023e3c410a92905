"""Torch-side plumbing around the binding: device buffers, streams, result download.

PyTorch is used for device memory and streams only; every step of the CTC path runs
in the HIP library.  Used by the GPU tests, the smoke check and the benchmark.
"""
from __future__ import annotations

import numpy as np
import torch

from . import ctc, workloads


def require_gpu() -> torch.device:
    if not torch.cuda.is_available():
        raise RuntimeError("a HIP device is required: the CTC path has no CPU fallback")
    return torch.device("cuda:0")


class DeviceBatch:
    """A CTCBatch with its activations resident in HBM plus output and workspace buffers."""

    def __init__(self, batch: workloads.CTCBatch, dtype: int = ctc.DTYPE_F32, device=None,
                 poison: bool = True):
        self.device = device or require_gpu()
        self.batch = batch
        self.dtype = dtype
        if dtype == ctc.DTYPE_F32:
            host = torch.from_numpy(np.ascontiguousarray(batch.logits, dtype=np.float32))
            self.x = host.to(self.device)
        else:
            bits = workloads.bf16_bits(batch.logits).view(np.int16)
            self.x = torch.from_numpy(bits).to(self.device).view(torch.bfloat16)
        self.grads = torch.empty_like(self.x)
        self.costs = torch.empty(batch.B, dtype=torch.float32, device=self.device)
        self.ws_bytes = ctc.workspace_size(batch.T, batch.B, batch.A, batch.label_lengths,
                                           batch.input_lengths, dtype)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=self.device)
        self.ws_ptr = (self.ws.data_ptr() + 255) // 256 * 256
        if poison:
            self.poison()

    def poison(self):
        """Fill outputs and workspace with NaN bit patterns so that stale data cannot pass."""
        self.ws.fill_(0xFF)
        self.grads.view(torch.uint8).fill_(0xFF)
        self.costs.fill_(float("nan"))

    def run(self, stream=None, kernel_ms=None):
        b = self.batch
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        ctc.loss_and_grad(self.x.data_ptr(), b.flat_labels, b.label_lengths, b.input_lengths,
                          b.T, b.B, b.A, b.blank, self.dtype, self.costs.data_ptr(),
                          self.grads.data_ptr(), self.ws_ptr, self.ws_bytes, s, kernel_ms)

    def run_loss(self, stream=None, kernel_ms=None):
        """Costs only (grads == NULL)."""
        b = self.batch
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        ctc.loss_and_grad(self.x.data_ptr(), b.flat_labels, b.label_lengths, b.input_lengths,
                          b.T, b.B, b.A, b.blank, self.dtype, self.costs.data_ptr(),
                          None, self.ws_ptr, self.ws_bytes, s, kernel_ms)

    def run_best_path(self, stream=None, kernel_ms=None):
        """Most probable alignment: scores go to self.costs, states to self.alignment [B,T]."""
        b = self.batch
        if getattr(self, "alignment", None) is None:
            self.alignment = torch.full((b.B, b.T), -7, dtype=torch.int32, device=self.device)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        ctc.best_path(self.x.data_ptr(), b.flat_labels, b.label_lengths, b.input_lengths,
                      b.T, b.B, b.A, b.blank, self.dtype, self.costs.data_ptr(),
                      self.alignment.data_ptr(), self.ws_ptr, self.ws_bytes, s, kernel_ms)

    def best_path_results(self):
        """(scores float32 [B], states int32 [B,T]) on the host, after synchronising."""
        torch.cuda.synchronize(self.device)
        return self.costs.cpu().numpy(), self.alignment.cpu().numpy()

    def results(self):
        """(costs float32 [B], grads float32 [T,B,A]) on the host, after synchronising."""
        torch.cuda.synchronize(self.device)
        costs = self.costs.cpu().numpy()
        if self.dtype == ctc.DTYPE_F32:
            grads = self.grads.cpu().numpy()
        else:
            grads = self.grads.float().cpu().numpy()
        return costs, grads


def run_batch(batch: workloads.CTCBatch, dtype: int = ctc.DTYPE_F32):
    db = DeviceBatch(batch, dtype)
    db.run()
    return db.results()


class DeviceMetaBatch:
    """Buffers for ctc_loss_and_grad_device: lengths and padded labels live on the GPU.

    Sized by bounds (T, B, A, max_label); `load` writes one CTCBatch of that shape into the
    same device buffers, so a recorded graph can be replayed on new contents.
    """

    def __init__(self, T, B, A, max_label, blank=0, dtype: int = ctc.DTYPE_F32, device=None):
        self.device = device or require_gpu()
        self.T, self.B, self.A, self.max_label, self.blank, self.dtype = T, B, A, max_label, blank, dtype
        tdtype = torch.float32 if dtype == ctc.DTYPE_F32 else torch.bfloat16
        self.x = torch.zeros((T, B, A), dtype=tdtype, device=self.device)
        self.grads = torch.empty_like(self.x)
        self.costs = torch.empty(B, dtype=torch.float32, device=self.device)
        self.labels = torch.zeros((B, max(max_label, 1)), dtype=torch.int32, device=self.device)
        self.label_lengths = torch.zeros(B, dtype=torch.int32, device=self.device)
        self.input_lengths = torch.zeros(B, dtype=torch.int32, device=self.device)
        self.status = torch.full((1,), -1, dtype=torch.int32, device=self.device)
        self.ws_bytes = ctc.workspace_size_device(T, B, A, max_label, dtype)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=self.device)
        self.ws_ptr = (self.ws.data_ptr() + 255) // 256 * 256

    def load(self, batch: workloads.CTCBatch, raw_labels=None):
        """Copies a batch into the device buffers (in place).  `raw_labels` [B, max_label] overrides
        the padded label matrix (to plant invalid entries)."""
        assert (batch.T, batch.B, batch.A) == (self.T, self.B, self.A)
        if self.dtype == ctc.DTYPE_F32:
            self.x.copy_(torch.from_numpy(np.ascontiguousarray(batch.logits, dtype=np.float32)))
        else:
            bits = workloads.bf16_bits(batch.logits).view(np.int16)
            self.x.copy_(torch.from_numpy(bits).view(torch.bfloat16))
        pad = np.zeros((self.B, max(self.max_label, 1)), dtype=np.int32)
        off = 0
        for b in range(self.B):
            L = int(batch.label_lengths[b])
            pad[b, :min(L, self.max_label)] = batch.flat_labels[off:off + L][:self.max_label]
            off += L
        if raw_labels is not None:
            pad = np.ascontiguousarray(raw_labels, dtype=np.int32)
        self.labels.copy_(torch.from_numpy(pad))
        self.label_lengths.copy_(torch.from_numpy(np.ascontiguousarray(batch.label_lengths, dtype=np.int32)))
        self.input_lengths.copy_(torch.from_numpy(np.ascontiguousarray(batch.input_lengths, dtype=np.int32)))

    def poison(self):
        self.ws.fill_(0xFF)
        self.grads.view(torch.uint8).fill_(0xFF)
        self.costs.fill_(float("nan"))
        self.status.fill_(-1)

    def run(self, stream=None, want_grad=True, kernel_ms=None):
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        ctc.loss_and_grad_device(self.x.data_ptr(), self.labels.data_ptr(), self.label_lengths.data_ptr(),
                                 self.input_lengths.data_ptr(), self.max_label, self.T, self.B, self.A,
                                 self.blank, self.dtype, self.costs.data_ptr(),
                                 self.grads.data_ptr() if want_grad else None, self.status.data_ptr(),
                                 self.ws_ptr, self.ws_bytes, s, kernel_ms)

    def results(self):
        """(status int, costs float32 [B], grads float32 [T,B,A]) on the host, after synchronising."""
        torch.cuda.synchronize(self.device)
        return int(self.status.item()), self.costs.cpu().numpy(), self.grads.float().cpu().numpy()
