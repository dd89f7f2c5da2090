"""Pins for the 4-bit dequantisation the oracle uses for the paper's intermediate-model format (oracle/quant.py)
and for the synthetic round-to-nearest quantiser that makes its inputs."""
import numpy as np
import torch

from oracle import quant as oquant
from paper_2510_26527_amd import synth


def test_worked_example():
    # one row, K = 256, two groups: codes 0..15 repeating; group 0: scale 0.5, zero 3; group 1: scale 2, zero 15
    q = (np.arange(256) % 16).astype(np.uint8)[None]
    codes = (q[:, 0::2] | (q[:, 1::2] << 4)).astype(np.uint8)
    assert np.array_equal(oquant.unpack_codes(codes), q)
    w = oquant.dequantize(codes, [[0.5, 2.0]], [[3, 15]])
    assert w.dtype == np.float32 and w.shape == (1, 256)
    assert w[0, 0] == -1.5 and w[0, 3] == 0.0 and w[0, 15] == 6.0
    assert w[0, 128] == -30.0 and w[0, 143] == 0.0 and w[0, 255] == 0.0


def test_grid_values_survive_a_round_trip():
    """Weights that already lie on a 4-bit grid are quantised to their own codes and come back exactly."""
    rng = np.random.default_rng(0)
    n, K = 24, 512
    q = rng.integers(0, 16, (n, K))
    q[:, ::128] = 0
    q[:, 1::128] = 15                    # every group spans the full code range, so min -> 0 and max -> 15
    zero = rng.integers(0, 16, (n, K // 128))
    scale = torch.tensor(rng.uniform(0.01, 0.05, (n, K // 128)), dtype=torch.float32).to(torch.bfloat16).float().numpy()
    w = np.repeat(scale, 128, 1) * (q - np.repeat(zero, 128, 1))
    codes, quant = synth.quantize_w4({"l0.wq": torch.tensor(w, dtype=torch.float32)})
    s, z = quant["l0.wq"]
    back = oquant.dequantize(codes["l0.wq"].numpy(), s.float().numpy(), z.numpy())
    assert np.abs(back - w).max() <= 1e-6 * np.abs(w).max()


def test_round_to_nearest_error_bound():
    rng = torch.Generator().manual_seed(1)
    w = torch.empty((64, 1024)).normal_(0, 0.02, generator=rng)
    codes, quant = synth.quantize_w4({"l3.w_down": w, "embed": w})
    assert codes["embed"] is w                                          # only projections are quantised
    s, z = quant["l3.w_down"]
    back = oquant.dequantize(codes["l3.w_down"].numpy(), s.float().numpy(), z.numpy())
    err = np.abs(back - w.numpy())
    bound = np.repeat(s.float().numpy(), 128, 1) * 0.51 + 1e-7          # half a step (the zero point is rounded too,
    frac = (err <= bound).mean()                                        # which can cost the extreme codes a little more)
    assert frac > 0.97 and err.max() <= np.repeat(s.float().numpy(), 128, 1).max() * 1.01
