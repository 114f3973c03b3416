"""Helpers shared by the GPU parity tests (no arithmetic of the method)."""
import numpy as np
import torch

from workloads import generators as gen

TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
# Tolerances of the parity gate: max |gpu - oracle| / max |oracle| against the fp64 oracle
# on dtype-rounded inputs.  fp16 / fp32 are the stated targets; bf16 (8 mantissa bits, unit
# round-off 2^-8 = 3.9e-3 applied once, to the fp32 accumulator) is gated like fp16.
TOL = {"f32": 1e-4, "f16": 2e-2, "bf16": 2e-2}


def to_dev(raw: np.ndarray, dtype: str) -> torch.Tensor:
    """Upload the raw storage array produced by generators.round_to_dtype."""
    if dtype == "bf16":
        return torch.from_numpy(raw.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(raw)).cuda()


def coords_dev(c: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(c, dtype=np.int32)).cuda()


def norm_err(got: torch.Tensor, ref: np.ndarray) -> float:
    g = got.detach().to(torch.float64).cpu().numpy()
    assert g.shape == ref.shape, (g.shape, ref.shape)
    assert np.isfinite(g).all()
    denom = np.abs(ref).max()
    if denom == 0:
        return float(np.abs(g).max())
    return float(np.abs(g - ref).max() / denom)


def make_layer(n_in, n_out, c_in, c_out, V, dtype, seed):
    """Features, weights and an output gradient: (values as float32, device tensor) each."""
    x32, xr = gen.features(n_in, c_in, dtype, seed)
    w32, wr = gen.weights(V, c_in, c_out, dtype, seed + 1)
    g32, gr = gen.features(n_out, c_out, dtype, seed + 2)
    return (x32, to_dev(xr, dtype)), (w32, to_dev(wr, dtype)), (g32, to_dev(gr, dtype))
