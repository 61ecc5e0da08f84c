"""The packed order of a decode step's weights, as include/molora.h states it element by
element, against the slab-by-slab rearrangement that the GPU tests compare molora_pack_w with
(numpy only: pins the two descriptions of the layout to each other, K tails included)."""
import numpy as np
import pytest


def packed_by_formula(W, gc):
    """Wp[16 s * d_out + g * n * gc + i * gc + c] = W[16 s + i][g * gc + c], n = rows of slab s."""
    d_in, d_out = W.shape
    Wp = np.empty(d_in * d_out, dtype=W.dtype)
    for s in range((d_in + 15) // 16):
        n = min(16, d_in - 16 * s)
        for g in range(d_out // gc):
            for i in range(n):
                at = 16 * s * d_out + g * n * gc + i * gc
                Wp[at:at + gc] = W[16 * s + i, g * gc:(g + 1) * gc]
    return Wp


def packed_by_slabs(W, gc):
    d_in, d_out = W.shape
    return np.concatenate([W[k0:k0 + 16].reshape(-1, d_out // gc, gc).transpose(1, 0, 2).ravel()
                           for k0 in range(0, d_in, 16)])


@pytest.mark.parametrize("d_in,d_out,gc", [(64, 64, 32), (72, 128, 32), (8, 64, 64), (200, 192, 64), (136, 8256 // 43, 64)])
def test_packed_order_formula_and_slab_form_agree(d_in, d_out, gc):
    W = np.arange(d_in * d_out, dtype=np.int64).reshape(d_in, d_out)
    a, b = packed_by_formula(W, gc), packed_by_slabs(W, gc)
    assert np.array_equal(a, b)
    assert np.array_equal(np.sort(a), np.arange(d_in * d_out)), "a permutation of W's elements"
    # slab s starts where it starts in W
    for s in range((d_in + 15) // 16):
        n = min(16, d_in - 16 * s)
        blk = a[16 * s * d_out:(16 * s + n) * d_out]
        assert np.array_equal(np.sort(blk), np.sort(W[16 * s:16 * s + n].ravel()))


def test_a_packed_b_keeps_every_slab_inside_one_adapter():
    """B [C][rank][d_out] packs as the [C * rank][d_out] matrix; with rank a multiple of 16 no
    slab of 16 rows straddles two adapters."""
    C, rank, d_out, gc = 3, 32, 64, 32
    B = np.arange(C * rank * d_out, dtype=np.int64).reshape(C, rank, d_out)
    p = packed_by_slabs(B.reshape(C * rank, d_out), gc)
    for c in range(C):
        seg = p[c * rank * d_out:(c + 1) * rank * d_out]
        assert np.array_equal(np.sort(seg), B[c].ravel())
