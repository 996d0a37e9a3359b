"""Host side of the IVFADC index (no GPU): the lookup count of the per-list Encoding Trees against the oracle's pointer
trie, entry merging, error codes."""
import numpy as np
import pytest

import oracle
from oracle import ivfadc
from oracle.trie import EncodingTree
import paper_1509_05186_amd as etf


def test_ivf_build_counts_match_the_pointer_trie_of_every_list():
    rng = np.random.default_rng(4)
    d, M, K, cells, N = 12, 6, 5, 7, 900
    cb = rng.normal(size=(M, K, d // M)).astype(np.float32)
    cent = rng.normal(size=(cells, d)).astype(np.float32) * 3
    x = (cent[rng.integers(0, cells, N)] + rng.normal(size=(N, d))).astype(np.float32)
    cl, codes = ivfadc.build(x, cent, cb)
    c = etf.Context(device=None)
    c.pq_set_codebooks(cb)
    c.ivf_set_coarse(cent)
    c.ivf_build(cl, codes)
    st = c.ivf_stats()
    want_lookups, want_entries, max_list, max_dup = 0, 0, 0, 0
    for j in range(cells):
        sub = codes[cl == j]
        if len(sub) == 0:
            continue
        uniq, counts = np.unique(sub, axis=0, return_counts=True)
        want_entries += len(uniq)
        max_list = max(max_list, len(uniq))
        max_dup = max(max_dup, int(counts.max()))
        want_lookups += EncodingTree(sub).stats()["lookups"]
    assert st["entries"] == want_entries and st["max_list"] == max_list and st["max_dup"] == max_dup
    assert st["tree_lookups"] == want_lookups
    assert st["flat_lookups"] == N * M and st["N"] == N and st["cells"] == cells


def test_ivf_host_error_paths():
    c = etf.Context(device=None)
    cb = np.zeros((2, 4, 3), dtype=np.float32)
    with pytest.raises(etf.EtfError):
        c._ck(c._lib.etf_ivf_set_coarse(c._h, None, 3))
    c.pq_set_codebooks(cb)
    with pytest.raises(etf.EtfError):
        c.ivf_stats()
    c.ivf_set_coarse(np.zeros((3, 6), dtype=np.float32))
    with pytest.raises(etf.EtfError) as e:
        c.ivf_build(np.array([0, 3], dtype=np.int32), np.zeros((2, 2), dtype=np.uint8))
    assert e.value.code == -1
    with pytest.raises(etf.EtfError):
        c.ivf_build(np.array([0, 1], dtype=np.int32), np.full((2, 2), 4, dtype=np.uint8))
    c.ivf_build(np.array([0, 1], dtype=np.int32), np.zeros((2, 2), dtype=np.uint8))
    with pytest.raises(etf.EtfError) as e:      # device entry point on a host-only context
        c._ck(c._lib.etf_ivf_upload(c._h, None, 0))
    assert e.value.code == -5
