"""A torch module around one RSR handle (the role the paper gives its RSRLinear layer in
System Overview, "Integration": a drop-in for a ternary linear layer whose weight is fixed after
preprocessing).  Argument marshalling only: the product runs in librsr."""
from __future__ import annotations

import torch

from . import binding as _b


class RsrLinear(torch.nn.Module):
    """y = scale * W x for a fixed int8 weight W [out_features][in_features] in {-1,0,+1}
    ({0,1} for the binary kind).  k = 0 lets the library choose the block height."""

    def __init__(self, weight: torch.Tensor, scale: float = 1.0, k: int = 0,
                 kind: int = _b.RSR_TERNARY_FUSED):
        super().__init__()
        self.out_features, self.in_features = weight.shape
        self.scale = float(scale)
        self.handle = _b.rsr_preprocess(weight, k, kind)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        if x.shape[-1] != self.in_features:
            raise ValueError("last dimension of x must be %d" % self.in_features)
        lead = x.shape[:-1]
        flat = x.reshape(-1, self.in_features)
        if flat.stride(-1) != 1:
            flat = flat.contiguous()
        if flat.shape[0] == 1:
            y = _b.rsr_matvec_ex(self.handle, flat[0], scale=self.scale).unsqueeze(0)
        else:
            y = _b.rsr_matvec_ex(self.handle, flat, scale=self.scale)
        return y.reshape(*lead, self.out_features)

    def extra_repr(self) -> str:
        return "in_features=%d, out_features=%d, k=%d, kind=%d" % (
            self.in_features, self.out_features, self.handle.k, self.handle.kind)
