"""Seeded synthetic inputs: attention shapes and accelerator descriptions.

Shared by the oracle-side tests and the GPU-side tests/benchmark.  This module
holds plain data and a random-number generator only -- none of the model's
arithmetic.  Everything is a dict of plain ints/floats; each side converts to
its own structs.

The workloads are shapes only (the paper's BERT-Base / GPT-3 / PaLM attention
layers are likewise just (heads, sequence length, head dim) triples), so these
synthetic shapes stand in for them.
"""
from __future__ import annotations

OBJ_ENERGY, OBJ_LATENCY, OBJ_LATENCY_THEN_ENERGY = 0, 1, 2

KiB = 1024
MiB = 1024 * 1024

_ENERGY = dict(e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0)   # pJ per word access / per MAC
_BW = dict(dram_bw=64.0, gb_bw=256.0)                          # bytes per cycle


def _wl(H, N, d, tiling_mode=0, B=1):
    return dict(B=B, H=H, N=N, d=d, word_bytes=2, tiling_mode=tiling_mode, c_softmax=10)


def _hw(pe, gb_bytes, rf_bytes, **kw):
    h = dict(pe_rows=pe, pe_cols=pe, n_arrays=1, rf_bytes=rf_bytes, gb_bytes=gb_bytes)
    h.update(_ENERGY)
    h.update(_BW)
    h.update(kw)
    return h


CONFIGS = {
    "tiny": dict(workload=_wl(1, 64, 32), hw=_hw(8, 16 * KiB, 64),
                 objectives=[OBJ_ENERGY]),
    "bert": dict(workload=_wl(12, 512, 64), hw=_hw(16, 256 * KiB, 256),
                 objectives=[OBJ_ENERGY, OBJ_LATENCY]),
    "prefill": dict(workload=_wl(32, 2048, 128), hw=_hw(32, 1 * MiB, 512),
                    objectives=[OBJ_LATENCY_THEN_ENERGY]),
    "long": dict(workload=_wl(32, 8192, 128, tiling_mode=1), hw=_hw(128, 8 * MiB, 1024),
                 objectives=[OBJ_ENERGY]),
}

def _chain(I, K, L, J, batch=1, tiling_mode=1):
    # GEMM chains carry no softmax between the operators
    return dict(batch=batch, I=I, K=K, L=L, J=J, word_bytes=2, tiling_mode=tiling_mode, c_softmax=0)


def conv_chain_as_gemms(hw_pixels, c_in, c_mid, c_out, k1, k2=1):
    """im2col of two back-to-back convolutions (the second one 1x1): rows = output pixels,
    reduction of the first = input channels x kernel window."""
    assert k2 == 1, "a second kernel larger than 1x1 is not a plain chain of two GEMMs"
    return hw_pixels, c_in * k1 * k1, c_mid, c_out


# an accelerator in the style of the paper's Accel. 1: 4 arrays of 32x32 PEs, 1 MiB buffer, 60 B/cycle
_ACCEL1 = dict(pe_rows=32, pe_cols=32, n_arrays=4, rf_bytes=512, gb_bytes=1 * MiB,
               e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=60.0, gb_bw=256.0)

# the shapes of the paper's Table V (two GEMMs and convolution chains)
CHAINS = {
    "mlp": dict(workload=_chain(768, 64, 384, 64), hw=_ACCEL1),
    "ffn": dict(workload=_chain(2048, 768, 3072, 768, tiling_mode=0), hw=_ACCEL1),
    "cc1": dict(workload=_chain(*conv_chain_as_gemms(112 * 112, 64, 192, 128, 3), tiling_mode=0), hw=_ACCEL1),
    "cc2": dict(workload=_chain(*conv_chain_as_gemms(56 * 56, 64, 64, 64, 1)), hw=_ACCEL1),
}

SWEEP_SEED = 0x260403446
_M64 = (1 << 64) - 1


class SplitMix64:
    """Steele, Lea & Flood's SplitMix64 generator (public-domain reference)."""

    def __init__(self, seed: int):
        self.s = seed & _M64

    def next(self) -> int:
        self.s = (self.s + 0x9E3779B97F4A7C15) & _M64
        z = self.s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
        return z ^ (z >> 31)

    def uniform(self) -> float:
        return (self.next() >> 11) / float(1 << 53)


def sweep_hw(n: int = 64, seed: int = SWEEP_SEED):
    """64 accelerators: PE array 8..128 squared, GB 64 KiB..16 MiB, RF 64 B..2 KiB,
    DRAM energy uniform in [100, 300) pJ."""
    rng = SplitMix64(seed)
    out = []
    for _ in range(n):
        pe = 8 << (rng.next() % 5)
        gb = (64 * KiB) << (rng.next() % 9)
        rf = 64 << (rng.next() % 6)
        e_dram = 100.0 + 200.0 * rng.uniform()
        out.append(_hw(pe, gb, rf, e_dram=e_dram))
    return out


def sweep_workloads():
    return [_wl(16, N, d) for N in (512, 1024, 4096, 16384) for d in (64, 128)]


def sweep_points():
    """All (workload, hw, objective) triples of the hardware sweep: 8 x 64 x 2."""
    pts = []
    for w in sweep_workloads():
        for h in sweep_hw():
            for obj in (OBJ_ENERGY, OBJ_LATENCY):
                pts.append((w, h, obj))
    return pts


def random_indices(space: int, n: int, seed: int):
    """n seeded candidate indices in [0, space)."""
    rng = SplitMix64(seed)
    return [rng.next() % space for _ in range(n)]
