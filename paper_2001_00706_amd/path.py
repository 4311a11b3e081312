"""`Path`: signatures of arbitrary intervals of a batch of paths in one group product each
(paper section 4.2, section 5.5 "arbitrary intervals" and "keeping the signature up-to-date").

Precomputed once: the signature of every prefix x_0..x_t (one stream-mode scan) and its inverse
(a signed permutation).  A query Sig(x_i..x_j) = Sig(x_0..x_i)^{-1} [x] Sig(x_0..x_j) is then one
strided `sig_combine` on rows of those two tensors, whatever the length of the path.  All
arithmetic runs in the HIP library; this class only keeps the tensors and computes row offsets.
"""
from __future__ import annotations

import torch

from . import binding


class Path:
    def __init__(self, path, depth: int):
        if path.dim() != 3 or path.shape[1] < 2:
            raise ValueError("path must have shape [B, L, d] with L >= 2")
        self.depth = int(depth)
        self.B, _, self.d = path.shape
        self.S = binding.sig_signature_channels(self.d, self.depth)
        self._last_point = path[:, -1].contiguous()
        # row t-1 = Sig(x_0..x_t), t = 1..L-1
        self._sig = [binding.sig_signature(path.contiguous(), self.depth, stream=True)]
        self._inv = [binding.sig_invert(self._sig[0], self.d, self.depth)]
        self._merge()

    def _merge(self):
        if len(self._sig) > 1:
            self._sig = [torch.cat(self._sig, dim=1)]
            self._inv = [torch.cat(self._inv, dim=1)]
        self.n = self._sig[0].shape[1]   # number of increments seen so far

    @property
    def length(self) -> int:
        """Points seen so far."""
        return self.n + 1

    def update(self, new_points):
        """Appends `new_points` `[B, M, d]`: the prefix signatures continue from the last one, using it as
        `initial` and the last point seen as the basepoint of the new piece."""
        if new_points.dim() != 3 or new_points.shape[0] != self.B or new_points.shape[2] != self.d:
            raise ValueError("new_points must have shape [B, M, d]")
        new_points = new_points.contiguous()
        last_sig = self._sig[0][:, -1].contiguous()
        more = binding.sig_signature(new_points, self.depth, stream=True, basepoint=self._last_point, initial=last_sig)
        self._sig.append(more)
        self._inv.append(binding.sig_invert(more, self.d, self.depth))
        self._last_point = new_points[:, -1].contiguous()
        self._merge()

    def signature(self, start: int = 0, end: int | None = None, out=None):
        """Signature of the points `start..end` inclusive (0-based; `end` defaults to the last point)."""
        end = self.n if end is None else end
        if not (0 <= start < end <= self.n):
            raise ValueError(f"need 0 <= start < end <= {self.n}")
        sig = self._sig[0]
        if out is None:
            out = torch.empty((self.B, self.S), dtype=sig.dtype, device=sig.device)
        row = self.n * self.S   # scalars between the same row of consecutive paths
        b_rows = sig.reshape(-1)[(end - 1) * self.S:]
        if start == 0:
            out.copy_(sig[:, end - 1])
            return out
        a_rows = self._inv[0].reshape(-1)[(start - 1) * self.S:]
        return binding.sig_combine_strided(a_rows, row, b_rows, row, self.B, self.d, self.depth, out, self.S)

    def logsignature(self, start: int = 0, end: int | None = None, mode: str = "words"):
        """Logsignature of the points `start..end` inclusive (sections 2.3, 4.3): `sig_log` of that interval's
        signature, then for mode "words" the coefficients of the Lyndon words ("expand" keeps every word)."""
        if mode not in ("words", "expand"):
            raise ValueError('mode must be "words" or "expand"')
        full = binding.sig_log(self.signature(start, end), self.d, self.depth)
        return full if mode == "expand" else binding.sig_lyndon_gather(full, self.d, self.depth)
