"""Pins of the score-reduction reference (no GPU needed): numbers worked out by hand, closed forms
through the attention oracle, and algebraic identities.  Which reading equals the paper's elided
formula stays unpinned; these pin each reading to its own stated definition."""
import numpy as np
import torch

import oracle
from oracle.reduce import RATIO_MEAN, RATIO_OF_SUMS, SPAN_MEAN, reduce_mass, valid_slots
from paper_2603_06588_amd import workloads as W


def test_hand_worked_numbers():
    # one sequence, two heads, one row, two spans: (a, b) = (0.2, 0.2) and (0.1, 0.7)
    m = np.array([[[[0.2, 0.2]], [[0.1, 0.7]]]])
    assert np.allclose(reduce_mass(m, RATIO_MEAN), [0.3125])          # (1/2 + 1/8) / 2
    assert np.allclose(reduce_mass(m, RATIO_OF_SUMS), [0.25])         # 0.15 / (0.15 + 0.45)
    assert np.allclose(reduce_mass(m, SPAN_MEAN), [[0.15, 0.45]])
    # weighted sum instead of the average; span order swapped
    assert np.allclose(reduce_mass(m, RATIO_MEAN, head_weights=[2.0, 4.0]), [1.5])       # 2/2 + 4/8
    assert np.allclose(reduce_mass(m, RATIO_MEAN, span_a=1, span_b=0), [0.6875])         # (1/2 + 7/8) / 2
    assert np.allclose(reduce_mass(m, SPAN_MEAN, head_weights=[1.0, -1.0]), [[0.1, -0.5]])
    # two rows, the second not selected
    m2 = np.array([[[[0.2, 0.2], [9.0, 9.0]], [[0.1, 0.7], [9.0, 9.0]]]])
    assert np.allclose(reduce_mass(m2, RATIO_MEAN, query_sel=[[5, 6]]), [0.3125])
    assert np.allclose(reduce_mass(m2, SPAN_MEAN, query_sel=[[5, 7]], cu_q_lens=[0, 6]), [[0.15, 0.45]])
    # zero denominators count as zero; nothing selected scores zero
    assert np.allclose(reduce_mass(np.zeros((1, 2, 1, 2)), RATIO_MEAN), [0.0])
    assert np.allclose(reduce_mass(np.zeros((1, 2, 1, 2)), RATIO_OF_SUMS), [0.0])
    assert np.allclose(reduce_mass(m2, RATIO_MEAN, query_sel=[[3, 3]]), [0.0])


def test_valid_slots():
    assert list(valid_slots(0, 4, None, None)) == [0, 1, 2, 3]
    assert list(valid_slots(0, 4, [[2, 5]], [0, 10])) == [0, 1, 2]
    assert list(valid_slots(0, 4, [[2, 9]], [0, 10])) == [0, 1, 2, 3]      # capped by NQ
    assert list(valid_slots(0, 4, [[8, 12]], [0, 10])) == [0, 1]           # capped by n
    assert list(valid_slots(0, 4, [[-2, 3]], [0, 10])) == [2, 3]           # rows before the chunk: slots 0, 1 unused
    assert list(valid_slots(0, 4, [[6, 2]], [0, 10])) == []


def test_uniform_attention_gives_length_ratio():
    # Q = 0: every probability is 1 / (pos + 1), so with both spans inside the horizon the focus
    # ratio is |a| / (|a| + |b|) whatever the heads, rows and weights
    lens = [90, 77]
    gen = torch.Generator().manual_seed(3)
    spans = [[(4, 24), (30, 70)], [(0, 10), (10, 40)]]
    b = W.build_paged("ratio", lens, lens, 4, 2, 16, torch.float32, 1.0, gen, [0, 2, 3],
                      [(L - 3, L) for L in lens], spans, max_sel_q=3, max_spans=2)
    b.q.zero_()
    _, mass = oracle.attn_probe_batch(b)
    want = [20 / 60, 10 / 40]
    for mode in (RATIO_MEAN, RATIO_OF_SUMS):
        got = reduce_mass(mass.numpy(), mode, query_sel=b.query_sel.tolist(), cu_q_lens=b.cu_q_lens.tolist())
        assert np.allclose(got, want, atol=1e-12)
    w = [0.2, 0.3, 0.5]
    assert np.allclose(reduce_mass(mass.numpy(), RATIO_MEAN, head_weights=w), want, atol=1e-12)
    # span means: row at position pos sees |span| / (pos + 1)
    sm = reduce_mass(mass.numpy(), SPAN_MEAN)
    for i, L in enumerate(lens):
        for r, (a, e) in enumerate(spans[i]):
            assert abs(sm[i, r] - np.mean([(e - a) / (pos + 1) for pos in range(L - 3, L)])) < 1e-12


def test_identities():
    rng = np.random.default_rng(0)
    m = rng.random((5, 4, 3, 6))
    w = rng.random(4)
    sel = [[0, 3], [1, 3], [0, 1], [2, 2], [-1, 2]]
    base = reduce_mass(m, SPAN_MEAN, query_sel=sel, head_weights=w)
    # linear in the weights; accumulate adds; negated weights cancel
    assert np.allclose(reduce_mass(m, SPAN_MEAN, query_sel=sel, head_weights=2 * w), 2 * base)
    twice = reduce_mass(m, SPAN_MEAN, query_sel=sel, head_weights=w, scores_in=base)
    assert np.allclose(twice, 2 * base)
    assert np.allclose(reduce_mass(m, SPAN_MEAN, query_sel=sel, head_weights=-w, scores_in=base), 0.0)
    # identical heads: any weights summing to one give the single-head value
    same = np.repeat(m[:, :1], 4, axis=1)
    one = reduce_mass(same[:, :1], RATIO_MEAN, 1, 4, query_sel=sel)
    assert np.allclose(reduce_mass(same, RATIO_MEAN, 1, 4, query_sel=sel, head_weights=w / w.sum()), one)
    # the two ratio readings agree when a + b is the same for every head and row
    k = m.copy()
    k[..., 1] = 0.9 - k[..., 0] * 0.5
    k[..., 0] *= 0.5
    assert np.allclose(reduce_mass(k, RATIO_MEAN, query_sel=sel), reduce_mass(k, RATIO_OF_SUMS, query_sel=sel))
    # a ratio and its complement sum to one where something is selected
    r1 = reduce_mass(m, RATIO_MEAN, 0, 1, query_sel=sel)
    r2 = reduce_mass(m, RATIO_MEAN, 1, 0, query_sel=sel)
    assert np.allclose((r1 + r2)[[0, 1, 2, 4]], 1.0) and (r1 + r2)[3] == 0.0
