"""What the matrix units sustain on different operand values (measurement support).

    python -m paper_2211_16270_amd.mfma_probe [fp8]

Runs the library's MFMA-only loop (rnnt_debug_mfma_loop: 32x32x16 bf16, no memory access inside the loop) with
one and two waves per SIMD on four kinds of operand values and prints the rate of each next to the published
dense bf16 peak.  The operands the transducer kernels multiply (tanh outputs, weights ~ N(0, 1/H), softmax
gradients) are "random bf16" in this sense.
"""
from __future__ import annotations

import numpy as np

PEAK_TFLOPS = 2500.0


def patterns():
    rng = np.random.Generator(np.random.PCG64(2211))
    n = 32 * 64 * 8
    sign = rng.integers(0, 2, n, dtype=np.uint16) << 15
    expo = (118 + rng.integers(0, 8, n, dtype=np.uint16)) << 7          # magnitudes 2^-9 .. 2^-2
    mant = rng.integers(0, 128, n, dtype=np.uint16)
    return [("zeros", np.zeros(n, dtype=np.uint16)),
            ("ones", np.full(n, 0x3F80, dtype=np.uint16)),
            ("random, 3 mantissa bits", sign | np.uint16(122 << 7) | (mant & 0x70)),
            ("random bf16", sign | expo | mant)]


def main():
    import torch
    from . import binding as Bd

    assert torch.cuda.is_available(), "needs a GPU"
    iters = 20000
    print(f"# MFMA-only loop, v_mfma_f32_32x32x16_bf16, {iters} iterations of 16 MFMAs per wave, 256 compute units")
    print("# operand values, waves per SIMD, ms per launch, TFLOP/s, fraction of the published 2.5 PFLOP/s")
    out = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    for name, bits in patterns():
        frags = torch.from_numpy(bits.view(np.int16).copy()).cuda().view(torch.bfloat16)
        for wgs in (256, 512):
            best = None
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                st = Bd.rnnt_debug_mfma_loop(frags, out, wgs, iters)
                e1.record()
                assert st == 0, st
                e1.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None else min(best, ms)
            tf = 2.0 * 32 * 32 * 16 * 16 * iters * 4 * wgs / (best * 1e-3) / 1e12
            print(f"{name}, {wgs // 256}, {best:.2f}, {tf:.0f}, {tf / PEAK_TFLOPS:.3f}", flush=True)


def main_fp8():
    """The same for the fp8 (e4m3) MFMA 32x32x64 against the published 5.0 PFLOP/s."""
    import torch
    from . import binding as Bd

    rng = np.random.Generator(np.random.PCG64(2212))
    n = 32 * 64 * 32
    rnd = rng.integers(0, 256, n, dtype=np.uint8)
    rnd = np.where((rnd & 0x7F) == 0x7F, rnd & 0xF0, rnd).astype(np.uint8)          # no NaN encodings
    mid = ((rng.integers(0, 2, n, dtype=np.uint8) << 7) | ((4 + rng.integers(0, 6, n, dtype=np.uint8)) << 3)
           | rng.integers(0, 8, n, dtype=np.uint8)).astype(np.uint8)                 # magnitudes 2^-3 .. 2^2
    iters = 10000
    print(f"# MFMA-only loop, v_mfma_f32_32x32x64_f8f6f4 (e4m3), {iters} iterations of 16 MFMAs per wave, 256 compute units")
    print("# operand values, waves per SIMD, ms per launch, TFLOP/s, fraction of the published 5.0 PFLOP/s")
    out = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    for name, bits in [("zeros", np.zeros(n, dtype=np.uint8)), ("ones", np.full(n, 0x38, dtype=np.uint8)),
                       ("random e4m3, exponents 4..9", mid), ("random bytes", rnd)]:
        frags = torch.from_numpy(bits.copy()).cuda()
        for wgs in (256, 512):
            best = None
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                st = Bd.rnnt_debug_mfma_loop_fp8(frags, out, wgs, iters)
                e1.record()
                assert st == 0, st
                e1.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None else min(best, ms)
            tf = 2.0 * 32 * 32 * 64 * 16 * iters * 4 * wgs / (best * 1e-3) / 1e12
            print(f"{name}, {wgs // 256}, {best:.2f}, {tf:.0f}, {tf / 5000.0:.3f}", flush=True)


if __name__ == "__main__":
    import sys
    main()
    if "fp8" in sys.argv[1:]:
        main_fp8()
