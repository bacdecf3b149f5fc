"""nn.Linear-shaped front of the K-contiguous entry (paper, Section IV-D: the LLM case study replaces the dense
projections of the feed-forward block by block-sparse products C = W X^T with activations stored tokens x hidden).

Argument marshalling only: a SparseLinear owns a BCSR handle of its weight and forwards device pointers to
asp_spmm_xt; nothing is computed here.  Inputs and outputs are torch tensors (bf16 carried as int16 or bfloat16)
used as device memory."""
from __future__ import annotations

from . import binding as asp


class SparseLinear:
    """y[N x out_features] = x[N x in_features] x W^T with W (out_features x in_features) block-sparse bf16."""

    def __init__(self, out_features, in_features, row_ptr, col_idx, values, block=128):
        self.out_features, self.in_features, self.block = out_features, in_features, block
        self.handle = asp.asp_create_from_csr("bcsr", "bf16", block, block, out_features, in_features, row_ptr, col_idx,
                                              values)

    def __call__(self, x, out, stream=None):
        """x: [N, in_features], out: [N, out_features], contiguous 2-byte device tensors; out is overwritten.
        stream: a hipStream_t value; None = torch's current stream on x's device."""
        if x.shape[1] != self.in_features or out.shape != (x.shape[0], self.out_features):
            raise ValueError("shape mismatch: x %s, out %s" % (tuple(x.shape), tuple(out.shape)))
        if x.element_size() != 2 or out.element_size() != 2 or not x.is_contiguous() or not out.is_contiguous():
            raise ValueError("x and out must be contiguous bf16 (2-byte) tensors")
        if stream is None:   # the stream that x was (or is being) produced on, not the NULL stream
            import torch
            stream = torch.cuda.current_stream(x.device).cuda_stream
        asp.asp_spmm_xt(self.handle, x.data_ptr(), out.data_ptr(), x.shape[0], stream)
        return out

    def close(self):
        if self.handle is not None:
            asp.asp_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
