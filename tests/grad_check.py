"""Gradient comparison shared by the GPU parity tests (no GPU code here: numpy only).

A gradient tensor g[..., N, D] from the HIP path is compared with the fp64 oracle's r at three
granularities, so that one wrong row, one wrong 32-row block or a wrong tail cannot hide inside a
whole-head norm:

  1. relative Frobenius error of every head             <= 3e-2   (the stated tolerance)
  2. relative Frobenius error of every 32-row block     <= 3e-2   (tiles of the kernels are multiples of 32 rows)
  3. every element: |g - r| <= 2^-6 |r| + 0.15 rms(r over the element's 32-row block)

(3) allows four bf16 ulps of relative error plus an absolute floor.  The floor is what the method's own
roundings need, not slack for the kernel: Delta_i = sum_d dO_id O_id is formed from the bf16 O of the
forward pass, so it carries an error of about 2^-9 |dO_i| |O_i|, which enters dS_ij = P_ij (dP_ij - Delta_i)
undamped where dP_ij - Delta_i cancels.  For the first rows of a causal problem (one or two keys, large
P) that moves single elements of dQ by several per cent; a numpy model of the bf16 roundings (O, P, dS)
puts the worst element at 0.04 block-rms and single rows at up to 10 % relative error, while 32-row
blocks stay within 0.4 %.  So rows are not held to a relative bound of their own; a lost, stale or
garbage row moves its elements by about their own size and fails (3), and anything systematic fails (2).
The floor is local to the block because the gradients of a causal problem shrink towards the last keys:
a floor taken from the whole head would let a wrong last row through.
"""
import numpy as np

GRAD_RELF = 3e-2
BLOCK_ROWS = 32
ELEM_REL = 2.0 ** -6
ELEM_ABS_RMS = 0.15


def relf(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def check_head(g, r, tag):
    """g, r: [N, D] float64 arrays of one head."""
    assert g.shape == r.shape, (tag, g.shape, r.shape)
    assert np.isfinite(g).all(), (tag, "non-finite")
    nr = np.linalg.norm(r)
    if nr == 0.0:            # (a single query attending to a single key: dQ = dK = 0 exactly)
        assert np.abs(g).max() <= 1e-6, (tag, "expected zeros", np.abs(g).max())
        return
    e = float(np.linalg.norm(g - r) / nr)
    assert e <= GRAD_RELF, (tag, "head relF", e)
    n = r.shape[0]
    rms = nr / np.sqrt(r.size)
    for r0 in range(0, n, BLOCK_ROWS):
        rb, gb = r[r0:r0 + BLOCK_ROWS], g[r0:r0 + BLOCK_ROWS]
        nb = np.linalg.norm(rb)
        if nb == 0.0:        # (causal, more keys than queries: keys nobody sees)
            assert np.abs(gb).max() <= 1e-6 * max(rms, 1.0), (tag, "expected a zero block", r0)
            continue
        eb = float(np.linalg.norm(gb - rb) / nb)
        assert eb <= GRAD_RELF, (tag, "block relF", r0, eb)
        bound = ELEM_REL * np.abs(rb) + ELEM_ABS_RMS * nb / np.sqrt(rb.size)
        bad = np.abs(gb - rb) > bound
        if bad.any():
            i = np.argwhere(bad)[0]
            raise AssertionError((tag, "element", (r0 + int(i[0]), int(i[1])), float(gb[tuple(i)]), float(rb[tuple(i)]),
                                  "count in block", int(bad.sum())))


def check_grad(g, r, tag):
    """g, r: [..., N, D] float64 arrays; every leading index is one head."""
    assert g.shape == r.shape, (tag, g.shape, r.shape)
    lead = g.shape[:-2]
    g2 = g.reshape((-1,) + g.shape[-2:])
    r2 = r.reshape((-1,) + r.shape[-2:])
    for i in range(g2.shape[0]):
        idx = np.unravel_index(i, lead) if lead else ()
        check_head(g2[i], r2[i], (tag,) + tuple(int(x) for x in idx))
