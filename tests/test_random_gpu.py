"""Seeded random shapes with integer-valued inputs: every kernel family and tile configuration must
reproduce the oracle bit for bit and leave the guard bands around a misplaced output buffer alone.

(The shapes are drawn so that all of a case runs in well under a second; larger one-off runs of the
same kind, several thousand launches per family, found no mismatch either.)
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_1705_10591_amd as dconv

pytestmark = pytest.mark.gpu


def _check(run, want, what, rng):
    total = want.size
    g = int(rng.integers(0, 40))                           # start anywhere within a line
    buf = torch.full((total + 2048 + g,), float("nan"), device="cuda")
    out = buf[1024 + g:1024 + g + total].view(want.shape)
    try:
        run(out)
    except dconv.DconvError as e:
        assert e.status == dconv.STATUS_UNSUPPORTED, what
        return 0
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), want, err_msg=what)
    assert torch.isnan(buf[:1024 + g]).all() and torch.isnan(buf[1024 + g + total:]).all(), what
    return 1


def test_special_case_kernel_random_batches_and_channels():
    rng = np.random.default_rng(1705_10591)
    ran = 0
    for it in range(40):
        C = int(rng.choice([1, 1, 2, 3, 4]))
        F = int(rng.integers(1, 12 if C == 1 else 6))
        N = int(rng.integers(1, 5))
        H = int(rng.integers(F, F + 16))
        W = max(F, int(rng.choice([rng.integers(F, 64), rng.integers(64, 420), rng.integers(420, 1100)])))
        K = int(rng.choice([1, 3, 16, 31, 33, 64, 70, 129]))
        if N * K * (H - F + 1) * (W - F + 1) * C * F * F > 1.5e8:
            K = 8
        x, f = wl.integer_case(5000 + it, N, C, H, W, K, F)
        acc, _, _ = oracle.general(x, f)
        xd, fd = torch.from_numpy(x).cuda(), torch.from_numpy(f).cuda()
        for v in [dconv.VARIANT_AUTO, dconv.VARIANT_SPECIAL_CASE] + \
                 [dconv.VARIANT_SPECIAL_CASE_CFG0 + i for i in range(dconv.tile_config_count(True))]:
            what = f"N,C,H,W,K,F={(N, C, H, W, K, F)} variant {v:#x}"
            print(what, flush=True)
            ran += _check(lambda out: dconv.dconv_general(xd, fd, out=out, variant=v),
                          acc.astype(np.float32), what, rng)
    assert ran > 200


def test_short_data_types_random_shapes_layouts_and_configurations():
    rng = np.random.default_rng(1705_10592)
    ran = 0

    def blocked(a, cb):          # [X][C][A][B] -> [X][C/cb][A][B][cb]
        X, C, A, B = a.shape
        return np.ascontiguousarray(a.reshape(X, C // cb, cb, A, B).transpose(0, 1, 3, 4, 2))

    for it in range(30):
        kind = str(rng.choice(["bf16", "f16", "i8"]))
        cb = 32 if kind == "i8" else 16
        C = cb * int(rng.integers(1, 4))
        F = int(rng.integers(1, 8))
        N = int(rng.integers(1, 4))
        H = int(rng.integers(F, F + 14))
        W = max(F, int(rng.choice([rng.integers(F, 40), rng.integers(40, 160)])))
        K = int(rng.choice([1, 5, 31, 64, 70, 130]))
        if kind == "i8":
            x = rng.integers(-128, 128, (N, C, H, W), dtype=np.int8)
            f = rng.integers(-128, 128, (K, C, F, F), dtype=np.int8)
            acc, _, _ = oracle.general(x.astype(np.float32), f.astype(np.float32))
            want, out_type = acc.astype(np.int32), torch.int32
        else:
            xf, ff = wl.integer_case(7000 + it, N, C, H, W, K, F)
            acc, _, _ = oracle.general(xf, ff)
            want, out_type = acc.astype(np.float32), torch.float32
            x, f = wl.to_16bit(xf, kind)[1], wl.to_16bit(ff, kind)[1]
        tt = {"i8": torch.int8, "f16": torch.float16, "bf16": torch.bfloat16}[kind]
        for bl in (False, True):
            xs, fs = (blocked(x, cb), blocked(f, cb)) if bl else \
                (np.ascontiguousarray(np.moveaxis(x, 1, -1)), np.ascontiguousarray(np.moveaxis(f, 1, -1)))
            if kind == "i8":
                xd, fd = torch.from_numpy(xs).cuda(), torch.from_numpy(fs).cuda()
            else:
                xd = torch.from_numpy(xs.view(np.int16)).view(tt).cuda()
                fd = torch.from_numpy(fs.view(np.int16)).view(tt).cuda()
            fn = dconv.dconv_general_i8 if kind == "i8" else dconv.dconv_general_half
            for v in [dconv.VARIANT_AUTO] + [dconv.VARIANT_TILED_CFG0 + i for i in range(5)]:
                what = f"{kind} N,C,H,W,K,F={(N, C, H, W, K, F)} blocked={bl} variant {v:#x}"
                print(what, flush=True)
                try:
                    out = fn(xd, fd, variant=v, blocked=bl)
                except dconv.DconvError as e:
                    assert e.status == dconv.STATUS_UNSUPPORTED, what
                    continue
                torch.cuda.synchronize()
                assert out.dtype == out_type
                np.testing.assert_array_equal(out.cpu().numpy(), want, err_msg=what)
                ran += 1
    assert ran > 200
