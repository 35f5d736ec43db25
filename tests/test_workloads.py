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
