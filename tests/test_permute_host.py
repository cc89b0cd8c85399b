"""Host-side logic of the general storage-order change: argument validation
(before any HIP call, so it runs without a GPU) and the canonical form the
library reduces a permutation to before it picks a kernel."""
import itertools

import numpy as np
import pytest

from paper_1610_03618_amd import binding as cm

PERMS = list(itertools.permutations(range(4)))
FAKE = 0x1000       # a non-null, 16-byte aligned address; invalid calls never dereference it


@pytest.mark.parametrize("dims", [(3, 5, 4, 7), (1, 5, 4, 7), (3, 1, 1, 7), (2, 3, 4, 1), (1, 1, 6, 1), (1, 1, 1, 1)])
def test_canonical_form_describes_the_same_permutation(dims):
    x = np.arange(int(np.prod(dims))).reshape(dims)
    for perm in PERMS:
        st, rank, cd, cp = cm.cnnmem_debug_canonical_permutation(dims, perm)
        assert st == 0 and 0 <= rank <= 4
        assert int(np.prod(cd)) == x.size if rank else x.size == 1
        assert sorted(cp) == list(range(rank))
        assert all(d > 1 for d in cd)
        want = x.transpose(perm).ravel()
        got = x.reshape(cd).transpose(cp).ravel() if rank else x.ravel()
        assert np.array_equal(got, want), (dims, perm)
        # nothing left to merge: no two neighbours of the destination are neighbours, in order, in the source
        assert all(cp[i + 1] != cp[i] + 1 for i in range(rank - 1))


def test_canonical_form_of_the_named_layouts():
    # NCHW -> CHWN is the 2-D transpose of [N][CHW]; NCHW -> NHWC a batch of [C][HW] transposes
    assert cm.cnnmem_debug_canonical_permutation((128, 96, 55, 55), (1, 2, 3, 0)) == (0, 2, [128, 290400], [1, 0])
    assert cm.cnnmem_debug_canonical_permutation((128, 96, 55, 55), (0, 2, 3, 1)) == (0, 3, [128, 96, 3025], [0, 2, 1])
    assert cm.cnnmem_debug_canonical_permutation((128, 96, 55, 55), (0, 1, 2, 3)) == (0, 1, [37171200], [0])
    # CHWN -> HWCN keeps N fastest: [C][HW][N] -> [HW][C][N]
    assert cm.cnnmem_debug_canonical_permutation((96, 55, 55, 128), (1, 2, 0, 3)) == (0, 3, [96, 3025, 128], [1, 0, 2])


@pytest.mark.parametrize("dims,perm", [
    ((0, 2, 2, 2), (0, 1, 2, 3)), ((2, 2, 2, -1), (0, 1, 2, 3)), ((2, 2, 2, 2), (0, 1, 1, 3)),
    ((2, 2, 2, 2), (0, 1, 2, 4)), ((2, 2, 2, 2), (-1, 1, 2, 3)),
])
def test_permute_rejects_invalid_arguments_on_host(dims, perm):
    assert cm.cnnmem_permute(FAKE, FAKE + 4096, dims, perm, stream=0) == 1
    assert cm.cnnmem_debug_canonical_permutation(dims, perm)[0] == 1


def test_permute_rejects_null_and_misaligned_pointers():
    assert cm.cnnmem_permute(None, FAKE, (2, 2, 2, 2), (0, 1, 2, 3), stream=0) == 1
    assert cm.cnnmem_permute(FAKE, None, (2, 2, 2, 2), (0, 1, 2, 3), stream=0) == 1
    assert cm.cnnmem_permute(FAKE + 2, FAKE + 4096, (2, 2, 2, 2), (0, 1, 2, 3), stream=0) == 1


@pytest.mark.parametrize("src,dst", [("NCHW", "NCH"), ("NCHW", "NCHWW"), ("NCHH", "NCHW"), ("NCHW", "nchw"),
                                     ("", "NCHW"), ("NCHW", "NCHX")])
def test_relayout_rejects_malformed_layouts_on_host(src, dst):
    assert cm.cnnmem_relayout(FAKE, FAKE + 4096, 2, 3, 4, 5, src, dst, stream=0) == 1


def test_relayout_rejects_bad_extents_on_host():
    assert cm.cnnmem_relayout(FAKE, FAKE + 4096, 0, 3, 4, 5, "NCHW", "NHWC", stream=0) == 1
    assert cm.cnnmem_relayout(FAKE, FAKE + 4096, 2, 3, 4, -5, "NCHW", "NHWC", stream=0) == 1
    assert cm.cnnmem_relayout(None, FAKE, 2, 3, 4, 5, "NCHW", "NHWC", stream=0) == 1
