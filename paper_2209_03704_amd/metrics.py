"""Work and traffic accounting for one layer (host arithmetic only).

"Useful" multiply-accumulates are the ones the segregated method of Section
3.3 performs: output (y, x) of parity (r, s) costs Ta(r) * Tb(s) taps per
(ci, co), with Ta(0) = ceil(n/2) and Ta(1) = floor(n/2) (the sub-kernel sizes
of Section 3.2; with an odd padding factor the two swap).  With E = ceil(M/2) even and O = floor(M/2) odd output
rows, the total is (E*ceil(n/2) + O*floor(n/2))^2 per (b, ci, co).  For even n
that is exactly a quarter of the conventional M^2 n^2 (Table 4); for odd n a
little less than a quarter.

"Algorithmic bytes" are what the method must move once: read in, read w,
write out.
"""
from __future__ import annotations

from .workloads import Layer

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0, "f16": 2500.0}
# fp32 on the vector ALUs: 256 CUs x 4 SIMDs x 32 multiply-adds per clock (packed pairs) x 2.4 GHz.
# Built without packed fp32 instructions (as this library is) a SIMD retires 16 per clock: half of it.
VALU_PEAK_TFLOPS = 157.3


def useful_macs(layer: Layer) -> int:
    M, n = layer.M, layer.n
    E, O = (M + 1) // 2, M // 2
    ce, fl = (n + 1) // 2, n // 2
    if layer.P & 1:          # odd padding factor: even output rows take the odd sub-kernel rows
        ce, fl = fl, ce
    return (E * ce + O * fl) ** 2 * layer.B * layer.Cin * layer.Cout


def conventional_macs(layer: Layer) -> int:
    return layer.M ** 2 * layer.n ** 2 * layer.B * layer.Cin * layer.Cout


def algorithmic_bytes(layer: Layer) -> int:
    eb = 2 if layer.dtype in ("bf16", "f16") else 4
    n_in = layer.B * layer.Cin * layer.N ** 2
    n_w = layer.Cout * layer.Cin * layer.n ** 2
    n_out = layer.B * layer.Cout * layer.M ** 2
    return eb * (n_in + n_w) + 4 * n_out


def upsampled_bytes(layer: Layer) -> int:
    """The (2N-1)^2 buffer the conventional method writes and re-reads."""
    eb = 2 if layer.dtype in ("bf16", "f16") else 4
    return eb * layer.B * layer.Cin * (2 * layer.N - 1) ** 2
