"""CPU-side checks of the dispatcher: which kernel and tile configuration a shape gets.

The paper fixes its tile sizes by exploring the design space per device (Sec. 5: 256 x 8 tiles
for the special case; Table 1 for the general case).  Here that exploration ended in rules that
pick one of the compiled configurations by shape; `dconv_tile_choice` answers with the rules'
pick from the shape alone, on the host, so the rules can be pinned without a GPU.  The pins below
are choices that were measured fastest (or within a few per cent of it) on MI355X; a change of a
rule that moves one of them has to come with a new measurement.
"""
import random

import pytest

import paper_1705_10591_amd as dconv

choice = dconv.tile_choice


# (H, W, K, F) -> configuration of the special-case kernel
SINGLE_PINS = [
    ((4096, 4096, 64, 5), 0),     # 512 x 4 tiles: the benchmark's headline shape
    ((4096, 4096, 64, 3), 0),
    ((4096, 4096, 64, 7), 0),
    ((4096, 4096, 64, 11), 2),    # 512 x 8: fewer halo rows per output row for the largest filters
    ((2048, 2048, 64, 9), 2),
    ((2400, 1600, 128, 9), 6),    # wide tiles would load the CUs unevenly
    ((1440, 1600, 128, 8), 6),
    ((1024, 1024, 64, 9), 0),     # 508 wide tiles: two per CU, even
    ((1800, 1800, 64, 7), 0),
    ((256, 256, 16, 3), 8),       # 64 x 4 tiles: a workgroup for every CU
    ((768, 768, 32, 5), 6),       # one filter block: the smallest tile, passes of 32 pixels
    ((1024, 1024, 32, 7), 0),
    ((640, 640, 128, 5), 6),      # 128 x 4 divides the image more evenly than 256 x 2
    ((3000, 3000, 32, 8), 2),
    ((720, 1280, 32, 5), 6),
    ((4096, 4096, 16, 5), 9),     # 16-filter matrix-core blocks
    ((720, 1280, 16, 5), 10),
    ((512, 512, 32, 3), 5),
]

# (H, W, K, F): one image of one channel that runs on the general-case kernel (narrow or short
# images, large filters: measured 8 to 38 % faster there; 12 x 12 and beyond always)
SINGLE_ON_THE_GENERAL_KERNEL = [(1536, 1536, 64, 11), (1080, 1920, 64, 9), (720, 1280, 64, 9), (256, 256, 32, 5),
                                (600, 800, 64, 7), (900, 1600, 128, 11), (1280, 1280, 32, 8), (768, 768, 64, 8),
                                (1536, 1280, 96, 11), (64, 64, 128, 8), (224, 224, 64, 3), (512, 512, 8, 13),
                                (224, 320, 8, 10), (384, 384, 6, 8)]
# ... and shapes that stay on the special case's kernels: the paper's sweep, large images that
# its wide tiles divide evenly, few filters
SINGLE_ON_ITS_OWN_KERNELS = [(4096, 4096, 64, 1), (4096, 4096, 64, 11), (2048, 2048, 64, 11), (3000, 3000, 64, 11),
                             (1024, 1024, 64, 9), (1024, 1024, 32, 7), (2048, 2048, 64, 5), (512, 512, 64, 3),
                             (512, 512, 8, 7), (256, 256, 8, 5), (1920, 1080, 32, 3)]

# (N, C, H, W, K, F) -> tile shape of the general kernel (0: 64 x 128, 1: 64 x 256, 2: 32 x 256)
GENERAL_PINS = [
    ((64, 3, 224, 224, 64, 11), 1),
    ((32, 64, 56, 56, 64, 3), 0),        # 729 small tiles in one round on 768 slots
    ((32, 256, 28, 28, 512, 3), 1),
    ((64, 32, 32, 32, 32, 3), 2),        # up to 32 filters: no padded half block
    ((13, 64, 75, 75, 96, 3), 2),        # 96 filters: the last block of 64 is half padding
    ((19, 256, 48, 48, 160, 3), 2),
    ((128, 256, 28, 28, 256, 1), 0),     # 1x1 with many channels
    ((256, 32, 112, 112, 64, 1), 1),     # 1x1 with few channels on wide maps
    ((64, 512, 7, 7, 512, 3), 0),        # tiny maps
    ((108, 320, 30, 30, 128, 2), 0),     # 2x2 with many channels
    ((94, 8, 224, 224, 64, 2), 1),       # few multiply-adds per output: bound by the stores
    ((1, 512, 14, 14, 512, 3), 0),       # fewer tiles than CUs
]


@pytest.mark.parametrize("dims,cfg", SINGLE_PINS)
def test_special_case_configuration_by_shape(dims, cfg):
    H, W, K, F = dims
    assert choice(True, 1, 1, H, W, K, F) == cfg


def test_one_channel_on_the_general_kernel_by_shape():
    for (H, W, K, F) in SINGLE_ON_THE_GENERAL_KERNEL:
        assert choice(True, 1, 1, H, W, K, F) == dconv.CHOICE_GENERAL_CASE, (H, W, K, F)
        # (dconv_general with one image of one channel takes the same route and names the tile shape)
        assert 0 <= choice(False, 1, 1, H, W, K, F) < 3, (H, W, K, F)
    for (H, W, K, F) in SINGLE_ON_ITS_OWN_KERNELS:
        assert choice(True, 1, 1, H, W, K, F) >= 0, (H, W, K, F)
        assert choice(False, 1, 1, H, W, K, F) == dconv.CHOICE_SPECIAL_CASE, (H, W, K, F)


@pytest.mark.parametrize("dims,shape", GENERAL_PINS)
def test_general_tile_shape_by_shape(dims, shape):
    assert choice(False, *dims) == shape


def test_other_kernels_by_shape():
    # one filter, the paper's own weak spot (Sec. 5): the vector-ALU kernel
    assert choice(True, 1, 1, 4096, 4096, 1, 3) == dconv.CHOICE_FEW_FILTERS
    assert choice(True, 1, 1, 2048, 2048, 8, 3) == dconv.CHOICE_FEW_FILTERS
    assert choice(True, 1, 1, 768, 768, 16, 3) >= 0            # too small an image for sixteen
    assert choice(True, 1, 1, 3000, 3000, 12, 2) >= 0          # an output beyond the memory-side cache, no arithmetic
    assert choice(True, 1, 1, 3000, 3000, 6, 2) == dconv.CHOICE_FEW_FILTERS
    # small images (its tiles do not cover the chip): one or two filters, more on mid-sized images
    assert choice(True, 1, 1, 256, 256, 1, 3) == dconv.CHOICE_FEW_FILTERS
    assert choice(True, 1, 1, 128, 128, 2, 5) == dconv.CHOICE_FEW_FILTERS
    assert choice(True, 1, 1, 256, 256, 1, 7) == dconv.CHOICE_GENERAL_CASE   # (a small image, a large filter)
    assert choice(True, 1, 1, 256, 256, 3, 5) >= 0
    assert choice(True, 1, 1, 256, 256, 4, 3) >= 0
    assert choice(True, 1, 1, 512, 512, 4, 3) == dconv.CHOICE_FEW_FILTERS
    assert choice(True, 1, 1, 512, 512, 3, 5) >= 0
    assert choice(True, 1, 1, 640, 640, 1, 7) == dconv.CHOICE_FEW_FILTERS
    # filters beyond the compiled sides
    assert choice(True, 1, 1, 512, 512, 8, 13) == dconv.CHOICE_GENERAL_CASE
    assert choice(True, 1, 1, 512, 512, 8, 33) == dconv.CHOICE_SIMPLE
    assert choice(False, 4, 64, 56, 56, 64, 13) >= 0
    assert choice(False, 4, 64, 56, 56, 64, 33) == dconv.CHOICE_SIMPLE
    # dconv_general with one channel, or a few with small filters and a large output
    assert choice(False, 1, 1, 1024, 1024, 64, 3) == dconv.CHOICE_SPECIAL_CASE
    assert choice(False, 16, 1, 512, 512, 64, 3) == dconv.CHOICE_SPECIAL_CASE
    assert choice(False, 16, 3, 512, 512, 64, 3) == dconv.CHOICE_SPECIAL_CASE
    assert choice(False, 16, 3, 512, 512, 64, 7) >= 0
    # a few filters on many channels: the vector-ALU kernel of the general case, where it covers the chip
    assert choice(False, 8, 64, 224, 224, 3, 3) == dconv.CHOICE_FEW_FILTERS
    assert choice(False, 8, 16, 224, 224, 1, 7) == dconv.CHOICE_FEW_FILTERS
    assert choice(False, 1, 256, 128, 128, 3, 3) == 2            # a few tiles, many channels to walk
    assert choice(False, 1, 3, 112, 112, 1, 5) == dconv.CHOICE_FEW_FILTERS      # a few tiles, few channels
    assert choice(False, 4, 3, 28, 28, 3, 3) == dconv.CHOICE_FEW_FILTERS
    assert choice(False, 1, 64, 56, 56, 8, 5) >= 0
    assert choice(False, 64, 256, 38, 38, 4, 1) == 2             # a barrier per channel for very little work
    assert choice(False, 21, 8, 96, 640, 12, 5) == dconv.CHOICE_FEW_FILTERS      # (nine to sixteen filters: few channels)
    assert choice(False, 15, 3, 384, 384, 10, 3) == dconv.CHOICE_FEW_FILTERS
    assert choice(False, 8, 256, 56, 56, 16, 3) == 2             # sixteen filters on many channels
    assert choice(False, 8, 64, 224, 224, 17, 3) == 2            # seventeen filters


@pytest.mark.parametrize("args", [
    (True, 1, 1, 8, 8, 4, 9), (True, 2, 1, 64, 64, 4, 3), (True, 1, 2, 64, 64, 4, 3),
    (False, 0, 1, 8, 8, 1, 3), (False, 1, 1, 8, 8, 0, 3), (False, 1, 1, 8, 8, 1, 0),
    (False, 1, 1, 40000, 40000, 4, 3), (False, 64, 1024, 1024, 1024, 1, 3),
])
def test_invalid_shapes(args):
    assert choice(*args) == dconv.CHOICE_INVALID


def test_every_answer_is_a_configuration_or_a_named_choice():
    rng = random.Random(1705)
    named = {dconv.CHOICE_FEW_FILTERS, dconv.CHOICE_SPECIAL_CASE, dconv.CHOICE_SIMPLE, dconv.CHOICE_GENERAL_CASE}
    n_single, n_general = dconv.tile_config_count(True), dconv.tile_config_count(False)
    for _ in range(3000):
        H, W = rng.randint(1, 5000), rng.randint(1, 5000)
        K, F = rng.randint(1, 300), rng.randint(1, 36)
        c = choice(True, 1, 1, H, W, K, F)
        if F > min(H, W) or K * (H - F + 1) * (W - F + 1) > 2**31 - 1:
            assert c == dconv.CHOICE_INVALID
        else:
            assert c in named - {dconv.CHOICE_SPECIAL_CASE} or 0 <= c < n_single, (H, W, K, F, c)
            assert c != 7              # the width-matching ablation is never chosen by shape
            assert (F > 11) <= (c in (dconv.CHOICE_SIMPLE, dconv.CHOICE_GENERAL_CASE)), (H, W, K, F, c)
            assert (c == dconv.CHOICE_SIMPLE) == (F > 32), (H, W, K, F, c)
            assert (c == dconv.CHOICE_GENERAL_CASE) <= (K >= 9 or F >= 6), (H, W, K, F, c)
        N, C = rng.randint(1, 64), rng.randint(1, 600)
        H, W = rng.randint(1, 300), rng.randint(1, 300)
        c = choice(False, N, C, H, W, K, F)
        if F > min(H, W):
            assert c == dconv.CHOICE_INVALID
        elif c != dconv.CHOICE_INVALID:
            assert c in named or 0 <= c < 3, (N, C, H, W, K, F, c)
            assert 3 * 4 * 2 == n_general     # shapes x schedules x write-backs


def test_rules_that_hold_for_every_shape():
    rng = random.Random(10591)
    for _ in range(2000):
        N, C = rng.randint(1, 64), rng.randint(5, 600)
        H, W = rng.randint(12, 200), rng.randint(12, 200)   # (some too small for the filter drawn below)
        K, F = rng.randint(1, 600), rng.randint(2, 32)
        if F > min(H, W):
            continue
        c = choice(False, N, C, H, W, K, F)
        assert c >= 0 or (c == dconv.CHOICE_FEW_FILTERS and K <= 16 and F <= 7), (N, C, H, W, K, F, c)
        if K <= 32 and c >= 0:
            assert c == 2          # no 64-filter block that is half padding
        if K % 64 == 0:
            assert c != 2          # nothing to save with 32-filter blocks
