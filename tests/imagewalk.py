"""Test helper: reads the level-ordered index image that the library exports and evaluates it with
numpy, level by level, exactly as the image's documentation in include/etf.h describes it.  This is
a check of the host-side builder (array contents, parent links, rows), not an implementation the
library uses."""
import numpy as np


def arr(buf, off, count, dtype):
    return np.frombuffer(buf, dtype=dtype, count=count, offset=off)


def walk_image(ctx, lut):
    """Per-input-position distances from the image and a [M][K] float64 table.
    Returns (dist[N] in input order, lookups done)."""
    st = ctx.index_stats()
    lay = ctx.index_layout()
    buf = ctx.index_export()
    N, Nd, T = st["N"], st["n_distinct"], st["T"]
    enc_of_pos = arr(buf, lay.enc_of_pos, N, np.uint32)
    total = np.zeros(Nd, dtype=np.float64)
    lookups = 0
    for t, tr in enumerate(st["trees"]):
        c0, D, U = tr["chunks"][0], tr["D"], tr["L2"]
        leafp = np.full(U, np.nan)
        part_prev = None
        for l in range(D):
            nI, nL = tr["nI"][l], tr["nL"][l]
            if nI:
                code = arr(buf, lay.icode[t][l], nI, np.uint8)
                par = arr(buf, lay.iparent[t][l], nI, np.uint32)
                if l == 0:
                    assert np.all(par == 0xFFFFFFFF)
                    part = lut[c0 + l, code]
                else:
                    assert par.max() < len(part_prev) and np.all(np.diff(par.astype(np.int64)) >= 0)
                    part = part_prev[par] + lut[c0 + l, code]
                lookups += nI
            else:
                part = np.zeros(0)
            if nL:
                stride = lay.lstride[t][l]
                width = D - l
                rec = arr(buf, lay.lcodes[t][l], nL * stride, np.uint8).reshape(nL, stride)
                par = arr(buf, lay.lparent[t][l], nL, np.uint32)
                row = arr(buf, lay.lrow[t][l], nL, np.uint32)
                assert np.all(rec[:, width:] == 0)
                if l == 0:
                    assert np.all(par == 0xFFFFFFFF)
                    acc = np.zeros(nL)
                else:
                    assert par.max() < len(part_prev)
                    acc = part_prev[par].copy()
                for j in range(width):
                    acc = acc + lut[c0 + l + j, rec[:, j]]
                lookups += nL * width
                assert np.all(np.isnan(leafp[row]))
                leafp[row] = acc
            part_prev = part
        assert not np.any(np.isnan(leafp))
        if lay.leaf_of[t] < 0:          # a single tree without leaf payload: entry e is leaf e
            assert T == 1 and U == Nd
            total += leafp
        else:
            leaf_of = arr(buf, lay.leaf_of[t], Nd, np.uint32)
            total += leafp[leaf_of]
    if lay.eterm >= 0:                  # leaf payload: the entry's term, added last
        total = total + arr(buf, lay.eterm, Nd, np.float32).astype(np.float64)
        assert np.array_equal(arr(buf, lay.pterm, N, np.float32), arr(buf, lay.eterm, Nd, np.float32)[enc_of_pos])
    return total[enc_of_pos], lookups
