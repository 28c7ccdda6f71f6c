"""Pins of the oracle's morphological clean-up of the region partition (section "Adaptive Region Partition":
opening and closing make the two regions more continuous; Algorithm 1 applies erosion and dilation to cos > eta)."""
import numpy as np
import pytest
from scipy import ndimage

from oracle import regione_oracle as orc

SQUARE = np.ones((3, 3), dtype=bool)


@pytest.mark.parametrize("shape", [(1, 1), (1, 7), (5, 1), (8, 8), (16, 16), (13, 29)])
@pytest.mark.parametrize("density", [0.1, 0.5, 0.9])
def test_erosion_and_dilation_match_the_library_routines(shape, density):
    rng = np.random.default_rng(shape[0] * 100 + shape[1] + int(density * 10))
    m = rng.random(shape) < density
    # "cells outside the grid never decide" = erosion sees set cells outside, dilation sees clear cells outside
    assert np.array_equal(orc.erode3x3(m), ndimage.binary_erosion(m, structure=SQUARE, border_value=1))
    assert np.array_equal(orc.dilate3x3(m), ndimage.binary_dilation(m, structure=SQUARE, border_value=0))
    # ... which is the same as replicating the border cells outwards and using the textbook operators on the padded grid
    padded = np.pad(m, 1, mode="edge")
    assert np.array_equal(orc.erode3x3(m), ndimage.binary_erosion(padded, structure=SQUARE)[1:-1, 1:-1])
    assert np.array_equal(orc.dilate3x3(m), ndimage.binary_dilation(padded, structure=SQUARE)[1:-1, 1:-1])


def _clean(edited_2d):
    h, w = edited_2d.shape
    return orc.mask_cleanup(edited_2d.reshape(-1).astype(np.uint8), h, w).reshape(h, w).astype(bool)


def test_cleanup_hand_cases():
    base = np.zeros((12, 12), dtype=bool)
    base[3:9, 2:8] = True                      # a 6x6 edited rectangle
    assert np.array_equal(_clean(base), base)  # regions at least as large as the element on both sides survive
    noisy = base.copy()
    noisy[0, 10] = True                        # an isolated edited token among unedited ones: a hole of the unedited map, closed
    noisy[5, 5] = False                        # an isolated unedited token inside the edit: a speck of the unedited map, opened away
    assert np.array_equal(_clean(noisy), base)
    assert not _clean(np.zeros((5, 5), dtype=bool)).any()      # nothing edited stays nothing edited
    assert _clean(np.ones((5, 5), dtype=bool)).all()           # everything edited stays everything edited
    thin = np.zeros((9, 9), dtype=bool)
    thin[:, 4] = True                          # an edited line one token wide is a gap of the unedited map narrower than the element
    assert not _clean(thin).any()
    wide = np.ones((9, 9), dtype=bool)
    wide[:, 3:5] = False                       # an unedited strip two tokens wide cannot hold the 3x3 element: opened away
    assert _clean(wide).all()
    strip3 = np.ones((9, 9), dtype=bool)
    strip3[:, 3:6] = False                     # three wide: survives
    assert np.array_equal(_clean(strip3), strip3)


@pytest.mark.parametrize("seed", range(6))
def test_cleanup_properties_and_library_composition(seed):
    rng = np.random.default_rng(seed)
    h, w = int(rng.integers(4, 40)), int(rng.integers(4, 40))
    edited = rng.random((h, w)) < rng.choice([0.05, 0.3, 0.6, 0.95])
    got = _clean(edited)
    un = ~edited
    opened = ndimage.binary_dilation(ndimage.binary_erosion(un, structure=SQUARE, border_value=1), structure=SQUARE, border_value=0)
    closed = ndimage.binary_erosion(ndimage.binary_dilation(opened, structure=SQUARE, border_value=0), structure=SQUARE, border_value=1)
    assert np.array_equal(got, ~closed)
    # opening followed by closing is an idempotent filter: cleaning a cleaned partition changes nothing
    assert np.array_equal(_clean(got), got)
    # opening only removes unedited cells, closing only adds them back
    assert not (opened & ~un).any()
    assert not (opened & ~closed).any()
