"""The comparison helpers themselves (CPU): the variant written for very large databases accepts and rejects what
the general one does."""
import numpy as np
import pytest

from parity import assert_topk_matches, assert_topk_matches_identity


def test_identity_variant_agrees_with_general_check():
    rng = np.random.default_rng(0)
    n, k = 5000, 100
    for trial in range(20):
        ref = rng.gamma(4, 10, size=n)
        ref[rng.integers(0, n, 200)] = ref[rng.integers(0, n, 200)]          # exact ties
        order = np.lexsort((np.arange(n), ref))[:k]
        gi, gd = order.copy(), ref[order].astype(np.float32)
        assert_topk_matches(gi, gd, ref, np.arange(n), k)
        assert_topk_matches_identity(gi, gd, ref, k)
        planted = []
        bi, bd = gi.copy(), gd.copy()                                         # a far vector in place of the k-th
        bi[-1] = np.argmax(ref)
        bd[-1] = ref[bi[-1]]
        planted.append((bi, bd))
        bi, bd = gi.copy(), gd.copy()                                         # a wrong distance
        bd[3] = bd[3] * 1.001
        planted.append((bi, bd))
        bi, bd = gi.copy(), gd.copy()                                         # the same id twice
        bi[5] = bi[4]
        planted.append((bi, bd))
        for bi, bd in planted:
            with pytest.raises(AssertionError):
                assert_topk_matches(bi, bd, ref, np.arange(n), k)
            with pytest.raises(AssertionError):
                assert_topk_matches_identity(bi, bd, ref, k)
