"""Buffer management around the C ABI: allocates the code / range / sum / workspace tensors with
torch (device memory only) and calls the entry points.  No arithmetic of the method happens
here; ``codes_to_logical`` is an index permutation for inspection and tests."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


class LanceConv:
    """One 3x3 convolution layer computed as quantized Winograd F(m x m, 3 x 3)."""

    def __init__(self, N, C, H, W, K, pad=1, m=2, bits=8, flags=0, device="cuda:0", bits_w=None):
        """bits: width of the input codes; bits_w: of the filter codes (default: the same).
        With B.LANCE_LAYOUT_NHWC in flags x is [N][H][W][C] and y is [N][Ho][Wo][K]."""
        if bits_w is not None:
            flags |= B.LANCE_FILTER_BITS(bits_w)
        self.desc = B.make_desc(N, C, H, W, K, pad, m, bits, flags)
        self.sz = B.lance_query_sizes(self.desc)
        self.device = torch.device(device)
        s, dev = self.sz, self.device
        self.uq = torch.empty(s.uq_bytes, dtype=torch.int8, device=dev)
        self.u_range = torch.empty((s.E, 2), dtype=torch.float32, device=dev)
        self.u_rowsum = torch.empty((s.E, K), dtype=torch.int32, device=dev)
        self.workspace = torch.empty(s.conv_workspace_bytes, dtype=torch.uint8, device=dev)
        self.v_range = torch.empty((s.E, 2), dtype=torch.float32, device=dev)
        self.nhwc = bool(flags & B.LANCE_LAYOUT_NHWC)
        self.packed = bool(flags & B.LANCE_CODES_PACKED4)
        self.y = torch.empty((N, s.Ho, s.Wo, K) if self.nhwc else (N, K, s.Ho, s.Wo),
                             dtype=torch.float32, device=dev)
        self._staged = None

    # -- stage 1, once per set of weights ---------------------------------------------------
    def prepare_filters(self, w: torch.Tensor, stream=None) -> None:
        B.lance_filter_transform_q8(self.desc, w, self.uq, self.u_range, self.u_rowsum, stream)

    # -- stages 2-4 fused -------------------------------------------------------------------
    def forward(self, x: torch.Tensor, y: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        y = self.y if y is None else y
        B.lance_conv3x3_winograd_q8(self.desc, x, self.uq, self.u_range, self.u_rowsum,
                                    self.v_range, y, self.workspace, stream=stream)
        return y

    # -- stages 2, 3, 4 one by one (every intermediate kept) ----------------------------------
    def alloc_staged(self):
        if self._staged is None:
            s, dev = self.sz, self.device
            self._staged = dict(
                vq=torch.empty(s.vq_bytes, dtype=torch.int8, device=dev),
                v_colsum=torch.empty((s.E, s.P), dtype=torch.int32, device=dev),
                acc=torch.empty((s.E, self.desc.K, s.P), dtype=torch.int32, device=dev),
                y=torch.empty_like(self.y))
        return self._staged

    def forward_staged(self, x: torch.Tensor, stream=None) -> dict:
        st = self.alloc_staged()
        B.lance_input_transform_q8(self.desc, x, st["vq"], self.v_range, st["v_colsum"],
                                   self.workspace, stream=stream)
        B.lance_winograd_gemm_i8(self.desc, self.uq, st["vq"], st["acc"], stream)
        B.lance_output_transform_dq(self.desc, st["acc"], self.u_range, self.u_rowsum,
                                    self.v_range, st["v_colsum"], st["y"], stream)
        return st

    # -- layout helper ----------------------------------------------------------------------
    def codes_to_logical(self, codes: torch.Tensor, rows: int) -> np.ndarray:
        """Blocked/permuted codes [E][NB][rows][CB] -> plain [E][rows][Cp] (host numpy).  Packed
        codes ([E][NB][rows][CB/2], two to a byte as code + 8) are split into bytes first."""
        s = self.sz
        a = codes.detach().cpu().numpy()
        if self.packed:
            b = a.view(np.uint8).reshape(s.E, s.NB, rows, s.CB // 2)
            a = (np.concatenate([b & 0xF, b >> 4], axis=-1).astype(np.int16) - 8).astype(np.int8)
        a = a.reshape(s.E, s.NB, rows, s.CB)
        Q = s.CB // 4
        r = np.arange(s.CB)
        pos = r if self.nhwc else 4 * (r % Q) + r // Q
        a = a[:, :, :, pos]                       # now indexed by in-block channel r
        return np.ascontiguousarray(a.transpose(0, 2, 1, 3).reshape(s.E, rows, s.Cp))
