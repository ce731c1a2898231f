"""Element-by-element comparison of the HIP library's hops with the oracle's (bit-exact)."""
import numpy as np

FIELDS = ("mb_rowoff", "row_vertex", "rowptr", "col", "mb_coloff", "col_vertex")
P_FIELDS = ("p_off", "p_col", "p_cnt")


def assert_hops_equal(gpu_hops, ref_hops, with_p=False, what=""):
    assert len(gpu_hops) == len(ref_hops)
    for h, (g, r) in enumerate(zip(gpu_hops, ref_hops)):
        g = g.to_host() if hasattr(g, "to_host") else g
        assert (g.rows, g.nnz, g.ncols) == (r.rows, r.nnz, r.ncols), \
            "%s hop %d sizes %s vs oracle %s" % (what, h, (g.rows, g.nnz, g.ncols), (r.rows, r.nnz, r.ncols))
        # the own-column array exists exactly when the oracle's variant has it
        assert (getattr(g, "row_self", None) is None) == (getattr(r, "row_self", None) is None), \
            "%s hop %d: row_self present on one side only" % (what, h)
        extra = ("row_self",) if getattr(r, "row_self", None) is not None else ()
        for name in FIELDS + (P_FIELDS if with_p else ()) + extra:
            a, b = getattr(g, name), getattr(r, name)
            assert a.shape == b.shape, "%s hop %d %s: shape %s vs %s" % (what, h, name, a.shape, b.shape)
            if not np.array_equal(a, b):
                bad = np.nonzero(a != b)[0]
                raise AssertionError("%s hop %d %s: %d of %d differ, first at %d: %s vs oracle %s" % (
                    what, h, name, bad.size, a.size, bad[0], a[bad[0]], b[bad[0]]))


def slice_minibatch(hop, i):
    """The part of a stacked host hop that belongs to minibatch i, re-based to start at 0."""
    from oracle.bms_oracle import Hop
    r0, r1 = int(hop.mb_rowoff[i]), int(hop.mb_rowoff[i + 1])
    c0, c1 = int(hop.mb_coloff[i]), int(hop.mb_coloff[i + 1])
    e0, e1 = int(hop.rowptr[r0]), int(hop.rowptr[r1])
    out = Hop(rows=r1 - r0, nnz=e1 - e0, ncols=c1 - c0,
              mb_rowoff=np.array([0, r1 - r0], dtype=np.int64), row_vertex=hop.row_vertex[r0:r1],
              rowptr=hop.rowptr[r0:r1 + 1] - e0, col=hop.col[e0:e1],
              mb_coloff=np.array([0, c1 - c0], dtype=np.int64), col_vertex=hop.col_vertex[c0:c1])
    if getattr(hop, "p_off", None) is not None:
        p0, p1 = int(hop.p_off[i]), int(hop.p_off[i + 1])
        out.p_off = np.array([0, p1 - p0], dtype=np.int64)
        out.p_col, out.p_cnt = hop.p_col[p0:p1], hop.p_cnt[p0:p1]
    return out
