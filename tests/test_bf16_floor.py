"""What bf16 STORAGE alone costs, in the metric of the parity bar (CPU only).

The oracle's storage-rounding probe rounds every tensor that a bf16 implementation keeps in bf16 between two
contractions (normalised rows, q / k / v, softmax weights, attention and GELU outputs) and leaves all arithmetic in
float64: its distance from the exact oracle is the error no implementation with bf16 operands can avoid on that
input.  These tests pin the probe itself, show on a Flux-shaped stage (hidden 3072, 24 heads of 128, MLP 12288: the
real width, so the modulation vectors have their real size; fewer rows and layers so that it runs in under a minute)
that the floor crosses the 2e-2 bar between a conditioning std of 0.5 and 1, and tie the conditioning std of every
named bf16 workload to the full-size floors stored in tests/golden/bf16_floor.txt (written by
tests/golden/make_bf16_floor.py from the oracle alone).
"""
import os

import numpy as np
import pytest

import workloads as wl
from oracle.pf_oracle import StageOracle

BAR = 2e-2
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "bf16_floor.txt")


def test_round_to_bf16_is_round_to_nearest_even_with_8_significant_bits():
    rng = np.random.Generator(np.random.Philox(key=5))
    a = rng.standard_normal(200000).astype(np.float32)
    r = wl.round_to_bf16(a)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)                           # representable in bf16
    rel = np.abs(r.astype(np.float64) - a) / np.abs(a)
    assert rel.max() <= 2.0 ** -8 * (1 + 1e-6)                                    # half an ulp (2^-7) of an 8-bit significand
    assert 1.2e-3 < np.sqrt(np.mean(rel ** 2)) < 2.0e-3                          # ~ 2^-8 / sqrt(3) times the binade average
    # ties go to the even neighbour: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)
    assert list(wl.round_to_bf16(ties)) == [1.0, 1.0 + 2.0 ** -6]


def test_identity_probe_changes_nothing():
    cfg = wl.CONFIGS["C4s"]
    W, A = wl.make_weights(cfg), wl.make_activations(cfg)
    n = wl.patch_rows(cfg)
    outs = []
    for probe in (None, lambda t: t):
        orc = StageOracle(cfg, W, storage_round=probe)
        orc.kv_init(A["x_prev"], A["cond"], text=A["text"])
        outs.append(orc.patch_forward(A["x"][n:2 * n], A["cond"], 1))
    assert np.array_equal(outs[0], outs[1])


@pytest.fixture(scope="module")
def flux_shaped_floors():
    base = wl._cfg(kind=3, dtype="bf16", n_layers=3, hidden=3072, n_heads=24, head_dim=128, mlp_dim=12288,
                   seq_img=512, grid_h=16, grid_w=32, n_patches=4, text_len=32, seed=41)
    W = wl.make_weights(base)
    layers64, out = None, {}
    for std in (0.25, 0.5, 1.0):
        cfg = wl.variant(base, cond_std=std)
        A = wl.make_activations(cfg)
        n, p = wl.patch_rows(cfg), 3
        ys = []
        for probe in (None, wl.round_to_bf16):
            orc = StageOracle(cfg, W if layers64 is None else layers64, storage_round=probe)
            layers64 = orc.layers                      # the float64 copies are shared by all runs
            orc.kv_init(None)
            for l in range(cfg["n_layers"]):
                orc.set_kv(l, *wl.make_kv_fill(cfg, l))
            ys.append(orc.patch_forward(A["x"][p * n:(p + 1) * n], A["cond"], p))
        ref, got = ys
        rms = np.sqrt(np.mean(ref ** 2))
        out[std] = (float(np.max(np.abs(got - ref)) / rms), float(np.sqrt(np.mean((got - ref) ** 2)) / rms))
    return out


def test_flux_shaped_floor_crosses_the_bar_between_half_and_unit_conditioning_std(flux_shaped_floors):
    f = flux_shaped_floors
    print({k: (f"{v[0]:.3e}", f"{v[1]:.3e}") for k, v in f.items()})
    assert f[1.0][0] > BAR > f[0.5][0] > f[0.25][0]
    # the typical (rms) error is a few roundings of relative size 2^-8 / sqrt(3) ~ 2e-3 (partly averaged out by the
    # contractions) in a row, far below the bar;
    # the bar is reached by the tail: columns with a large gate carry errors many times the typical one
    for std in f:
        assert 5e-4 < f[std][1] < 4e-3 and f[std][0] > 6 * f[std][1]
    # three layers and 128 rows here; at the configured 7 layers and 2048 rows the floor is higher still (golden file)


def _golden():
    rows = {}
    for line in open(GOLDEN):
        fld = line.split()
        if len(fld) >= 5 and not line.startswith("#"):
            rows[(fld[0], float(fld[1]))] = (float(fld[2]), float(fld[3]))
    return rows


def test_workload_conditioning_std_follows_the_full_size_floors():
    """Every named bf16 workload draws its conditioning embedding at the largest of the listed stds (1, 0.5, 0.25) at
    which bf16 storage alone - the floor of its own full-size, full-depth call - takes at most two thirds of the 2e-2
    bar.  The remaining third is for what an implementation adds (fp32 instead of float64 arithmetic, its own rounding
    order) and for the spread of a maximum over millions of outputs between calls and realisations of the same
    rounding noise (the GPU tests see up to +-15 %)."""
    g = _golden()
    for name in ("C2", "C3", "C4", "C5"):
        stds = sorted({s for (n, s) in g if n == name}, reverse=True)
        assert 1.0 in stds, name
        ok = [s for s in stds if g[(name, s)][0] <= BAR * 2 / 3]
        assert ok, f"{name}: no listed conditioning std keeps the storage floor under two thirds of the bar"
        assert wl.CONFIGS[name]["cond_std"] == max(ok), (name, wl.CONFIGS[name]["cond_std"], g)
    # the Flux-scale stage is the one the format limits: its floor alone exceeds the bar at std 0.5 and 1
    assert g[("C4", 1.0)][0] > BAR and g[("C4", 0.5)][0] > BAR
