"""What the full-size parity data can and cannot see, shown on the CPU with a mistake planted
in the ORACLE's input (no kernel is involved).

At tens of thousands of N(0,1) keys the softmax is flat: the absolute bound (2e-2) cannot see
a dropped 16-key page at all, and the relative Frobenius bound (1e-2) sees it by a factor of
about five.  The probe data of the full-size GPU tests (helpers:
one planted key per page, aimed queries) and the peaked data (scaled queries) must turn such
mistakes into errors of O(1)."""
import numpy as np
import pytest
import torch

from oracle import attention
from helpers import (PROBE_GAIN, assert_rows_close, chunk_probe_targets, probe_tokens, probe_vectors)

Hq, Hkv, D = 8, 2, 64
SCALE = 1.0 / 8.0


def bf16(shape, seed):
    g = torch.Generator()
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32).to(torch.bfloat16).float().numpy()


def drop_page(K, V, page):
    """The planted mistake: page `page` of the sequence is skipped (its 16 keys are gone)."""
    keep = np.ones(len(K), bool)
    keep[16 * page:16 * page + 16] = False
    return K[keep], V[keep]


def decode_out(q, K, V):
    return attention.attention_rows(q[None], np.array([len(K) - 1]), K, V, SCALE)[0]


def test_flat_data_sees_a_dropped_page_only_barely_and_probes_see_it_plainly():
    """N(0,1) data at 32K keys: the output is itself a noisy average of size sqrt(e/n), so a
    dropped page does move the relative Frobenius error over the bar (by a factor of about
    five, measured here), while the absolute bound cannot see it.  With probe data the same
    dropped page moves the aimed output by O(1): both bounds fail, fifty times over."""
    n = 32769                                       # 2049 pages, the last one holds a single key
    K, V = bf16((n, Hkv, D), 1), bf16((n, Hkv, D), 2)
    q = bf16((Hq, D), 3)
    truth = decode_out(q, K, V)
    from helpers import parity_counts
    for page in (0, 1000, 2047):
        err, rel, _ = parity_counts(decode_out(q, *drop_page(K, V, page)), truth)
        assert err < 1e-2 and 1e-2 < rel < 0.15, (page, err, rel)     # the absolute bound is blind; the relative one sees it
    # probe data: one planted key per page, Hq pages aimed at per call
    tokens = probe_tokens(5, n)
    u = probe_vectors(5, len(tokens), D).float().numpy()
    Kp = K.copy()
    Kp[tokens] = (PROBE_GAIN * u)[:, None, :]
    for page in (0, 1000, 2047, 2048):
        call = page // Hq
        qp = q.copy()
        sel = np.arange(call * Hq, min(len(tokens), (call + 1) * Hq))
        qp[:len(sel)] = u[sel]
        truth = decode_out(qp, Kp, V)
        # the aimed head returns the V row of the planted token
        h = page - call * Hq
        assert np.abs(truth[h] - V[tokens[page], h // (Hq // Hkv)]).max() < 1e-2
        wrong = decode_out(qp, *drop_page(Kp, V, page))
        err, rel, _ = parity_counts(wrong[:len(sel)], truth[:len(sel)])
        assert err > 0.5 and rel > 0.2, (page, err, rel)              # O(1): fifty times the bar
        with pytest.raises(AssertionError):
            assert_rows_close(wrong[:len(sel)], truth[:len(sel)], "probe data, page %d dropped" % page)
        # ... and a page read twice in place of its neighbour shows as well
        Kd, Vd = Kp.copy(), V.copy()
        other = page - 1 if page > 0 else 1
        lo, cnt = 16 * page, min(16, n - 16 * page)
        Kd[lo:lo + cnt], Vd[lo:lo + cnt] = Kp[16 * other:16 * other + cnt], V[16 * other:16 * other + cnt]
        with pytest.raises(AssertionError):
            assert_rows_close(decode_out(qp, Kd, Vd)[:len(sel)], truth[:len(sel)], "probe data, page %d replaced" % page)


def test_peaked_data_sees_a_dropped_key_range():
    """Scaled queries: the weight of a row sits on a few keys scattered over the context, so a
    lost stretch of keys (a key range cut one page short, say) moves most rows by O(1)."""
    n = 4096
    K, V = bf16((n, Hkv, D), 11), bf16((n, Hkv, D), 12)
    q = bf16((Hq, D), 13) * 5.0
    truth = decode_out(q, K, V)
    keep = np.ones(n, bool)
    keep[1024:2048] = False                           # a quarter of the keys gone
    wrong = attention.attention_rows(q[None], np.array([int(keep.sum()) - 1]), K[keep], V[keep], SCALE)[0]
    with pytest.raises(AssertionError):
        assert_rows_close(wrong, truth, "peaked data, keys 1024..2047 dropped")
    assert np.abs(wrong - truth).max() > 0.3          # O(1), not O(1/n)
    # and a single lost key, if it is one of the few that carry a row: the top key of head 0
    scores = (K[:, 0, :] @ q[0]) * SCALE
    top = int(np.argmax(scores))
    keep = np.ones(n, bool)
    keep[top] = False
    one = attention.attention_rows(q[None], np.array([n - 2]), K[keep], V[keep], SCALE)[0]
    with pytest.raises(AssertionError):
        assert_rows_close(one[:1], truth[:1], "peaked data, the heaviest key of head 0 dropped")


def test_chunk_probes_reach_every_page_with_a_row_that_sees_it():
    C, ql = 1000, 96
    n = C + ql
    tokens = probe_tokens(9, n)
    rows, heads = chunk_probe_targets(C, ql, Hq, tokens)
    assert (rows >= 0).all() and len(set(zip(rows.tolist(), heads.tolist()))) == len(tokens)
    assert (C + rows >= tokens).all()                 # causality: the aimed row sees its planted key
    K, V = bf16((n, Hkv, D), 21), bf16((n, Hkv, D), 22)
    u = probe_vectors(9, len(tokens), D).float().numpy()
    K[tokens] = (PROBE_GAIN * u)[:, None, :]
    q = bf16((ql, Hq, D), 23)
    q[rows, heads] = u
    truth = attention.attention_chunk(q, K, V, C, SCALE)
    G = Hq // Hkv
    for p in (0, 31, 62, 63, len(tokens) - 1):        # context pages, the page the chunk starts in, its last page
        assert np.abs(truth[rows[p], heads[p]] - V[tokens[p], heads[p] // G]).max() < 1e-2
    # drop a context page: positions shift by 16, the probing row loses its key
    page = 31
    Kw, Vw = drop_page(K, V, page)
    wrong = attention.attention_chunk(q, Kw, Vw, C - 16, SCALE)
    with pytest.raises(AssertionError):
        assert_rows_close(wrong[rows, heads], truth[rows, heads], "chunk probes, page %d dropped" % page)
    # more pages than (row, head) pairs: the surplus is reported as not probed
    rows2, _ = chunk_probe_targets(100000, 4, 2, probe_tokens(1, 100004))
    assert (rows2 >= 0).sum() == 8 and (rows2[8:] == -1).all()
