"""The seeded input generators (no method arithmetic lives there): checks of their helpers."""
import numpy as np
import torch

import workloads as wl


def test_rounding_to_16_bit_types_matches_the_library_casts():
    """to_16bit against torch's CPU conversions (round to nearest even), ties and subnormals included."""
    rng = np.random.default_rng(5)
    a = np.concatenate([rng.standard_normal(4000).astype(np.float32) * np.float32(3.0),
                        np.float32([0.0, -0.0, 1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -9, 1.0 + 2.0 ** -11,
                                    1.0 + 3 * 2.0 ** -12, 6.0e-5, 1.0e-7, 65504.0, -8.0, 0.0589])])
    for kind, tt in (("f16", torch.float16), ("bf16", torch.bfloat16)):
        vals, bits = wl.to_16bit(a, kind)
        ref = torch.from_numpy(a).to(tt)
        assert np.array_equal(vals, ref.to(torch.float32).numpy())
        assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())


def test_integer_cases_are_representable_in_16_bit_types():
    x, f = wl.integer_case(3, 2, 16, 9, 9, 5, 3)
    for kind in ("f16", "bf16"):
        assert np.array_equal(wl.to_16bit(x, kind)[0], x) and np.array_equal(wl.to_16bit(f, kind)[0], f)


def test_bench_refuses_more_than_one_gpu():
    """This build shows one GPU's share; bench.py says so instead of running with --gpus above 1."""
    import subprocess
    import sys
    from pathlib import Path
    root = Path(__file__).resolve().parent.parent
    r = subprocess.run([sys.executable, str(root / "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_workload_tables_are_consistent():
    """Every benchmark workload has positive sizes, a filter that fits and a unique seed."""
    import workloads as wl
    allw = list(wl.CONFIGS.values()) + list(wl.S2_SWEEP.values()) + list(wl.PAPER_SWEEP.values())
    seeds = set()
    for w in allw:
        assert min(w.N, w.C, w.H, w.W, w.K, w.F) >= 1 and w.F <= min(w.H, w.W), w.name
        assert w.out_elems == w.N * w.K * (w.H - w.F + 1) * (w.W - w.F + 1), w.name
        assert w.flops == 2 * w.out_elems * w.C * w.F * w.F, w.name
        if w.name != "S2_F5":          # the sweep's 5x5 entry is S2 itself
            assert w.seed not in seeds or w.name.startswith("S2"), w.name
        seeds.add(w.seed)
