"""hook_span_mass (many spans, probe only) against the fp64 oracle (needs an MI355X)."""
import pytest
import torch

import oracle
from paper_2603_06588_amd import workloads as W
from helpers import MASS_ATOL as MASS_TOL

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _selected_rows(b):
    rows = []
    cu = b.cu_q_lens.tolist()
    for i in range(b.num_seqs):
        qb, qe = b.query_sel[i].tolist()
        n = cu[i + 1] - cu[i]
        rows += [cu[i] + t for t in range(max(qb, 0), min(qe, n, qb + b.max_sel_q))]
    return rows


def _check(b):
    from paper_2603_06588_amd import binding
    _, want = oracle.attn_probe_batch(b, rows=_selected_rows(b))
    bd = b.to(DEV)
    # both forms: split over keys and spans (scratch memory given), and one workgroup per row block
    for use_ws in (False, True):
        got = binding.hook_span_mass_batch(bd, use_workspace=use_ws)
        torch.cuda.synchronize()
        again = binding.hook_span_mass_batch(bd, use_workspace=use_ws)
        torch.cuda.synchronize()
        assert torch.equal(got, again)                               # reproducible bit for bit
        got = got.cpu().double()
        assert torch.isfinite(got).all()
        err = (got - want).abs().max().item()
        assert err <= MASS_TOL, (use_ws, err)
    return got, want


@pytest.mark.parametrize("d", [128, 64])
def test_span_mass_small_ragged(d):
    # 40 spans incl. overlapping, empty, clipped and out-of-range ones; rows straddle 16-row blocks;
    # a decode row, a chunk with prior context, an empty sequence, an empty selection
    lens, qlens = [333, 90, 64, 1000, 17], [333, 1, 0, 40, 17]
    b = W.random_batch(500 + d, lens, qlens, 8, 2, d, torch.bfloat16, std=1.0, num_probe_heads=3, max_sel_q=37,
                       max_spans=40)
    b.query_sel[4, 0], b.query_sel[4, 1] = 5, 5
    got, want = _check(b)
    assert want.abs().max() > 0.05


def test_span_mass_agrees_with_probe_kernels_on_few_spans():
    from paper_2603_06588_amd import binding
    b = W.c2_prefill_8b(shrink=4, peaked=True).to(DEV)
    _, m1 = binding.hook_attn_probe_batch(b)
    m2 = binding.hook_span_mass_batch(b)
    torch.cuda.synchronize()
    assert (m1 - m2).abs().max().item() <= 2e-5


@pytest.mark.parametrize("peaked", [False, True])
def test_span_mass_reranker_shape(peaked):
    b = W.c6_reranker(peaked=peaked, shrink=2)
    got, want = _check(b)
    # disjoint documents: the masses of one row cannot exceed 1 in total
    assert got.sum(-1).max() <= 1 + 1e-4


def test_span_mass_reranker_full_size_and_calibration():
    from paper_2603_06588_amd import binding
    from oracle.reduce import SPAN_MEAN, reduce_mass
    b = W.c6_reranker()
    got, want = _check(b)
    # document scores: mean over heads and question rows, minus a calibration pass (here: the
    # same prompts with other question tokens), entirely on the device
    bd = b.to(DEV)
    mass = binding.hook_span_mass_batch(bd)
    calib = b.to(DEV)
    calib.q = torch.roll(bd.q, 7, dims=0).contiguous()
    mass_c = binding.hook_span_mass_batch(calib)
    scores = binding.hook_reduce_mass(mass, 0, query_sel=bd.query_sel, cu_q_lens=bd.cu_q_lens)
    w = torch.full((b.probe_heads.numel(),), -1.0 / b.probe_heads.numel(), device=DEV)
    binding.hook_reduce_mass(mass_c, 0, query_sel=bd.query_sel, cu_q_lens=bd.cu_q_lens, head_weights=w,
                             scores=scores, accumulate=True)
    torch.cuda.synchronize()
    ref = reduce_mass(mass.cpu().numpy(), SPAN_MEAN, query_sel=b.query_sel.tolist(), cu_q_lens=b.cu_q_lens.tolist())
    ref = ref - reduce_mass(mass_c.cpu().numpy(), SPAN_MEAN, query_sel=b.query_sel.tolist(),
                            cu_q_lens=b.cu_q_lens.tolist())
    assert abs(scores.cpu().double().numpy() - ref).max() <= 4e-6


def test_span_mass_with_invalid_device_contents_completes():
    """Block ids, lengths, selections and spans that make no sense must not take the call outside
    its buffers; the valid sequences still come out right."""
    from paper_2603_06588_amd import binding
    b = W.random_batch(520, [200, 300, 150, 90], [200, 1, 150, 1], 8, 2, 128, torch.bfloat16, std=1.0,
                       num_probe_heads=3, max_sel_q=20, max_spans=12, poison=False)
    _, want = oracle.attn_probe_batch(b, rows=_selected_rows(b))
    bad = b.to(DEV)
    bad.seq_lens = bad.seq_lens.clone()
    bad.seq_lens[2] = 100                                   # n_i > L_i: skipped
    bad.block_table = bad.block_table.clone()
    bad.block_table[3] = 0x7FFFFFF0                         # out-of-range ids: clamped
    bad.key_spans = bad.key_spans.clone()
    bad.key_spans[1, 0, 0], bad.key_spans[1, 0, 1] = -2**31, 2**31 - 1
    bad.key_spans[1, 1, 0], bad.key_spans[1, 1, 1] = 2**31 - 1, -2**31
    for use_ws in (False, True):
        got = binding.hook_span_mass_batch(bad, use_workspace=use_ws).cpu().double()
        assert torch.isfinite(got).all()
    assert torch.isfinite(got).all()
    assert (got[0] - want[0]).abs().max() <= MASS_TOL
    assert (got[2] == 0).all()
    assert abs(float(got[1, 0, 0, 0]) - 1.0) <= MASS_TOL and float(got[1, 0, 0, 1]) == 0.0


@pytest.mark.parametrize("d", [128, 64])
def test_span_mass_over_an_8_bit_cache(d):
    """The same pass over E4M3 key bytes with one scale per kv head: both forms against the oracle, which
    dequantises every byte; and the attention call's own probe on the same batch agrees."""
    from paper_2603_06588_amd import binding
    lens, qlens = [333, 90, 64, 1000, 17], [333, 1, 0, 40, 17]
    b = W.random_batch(560 + d, lens, qlens, 8, 2, d, torch.bfloat16, std=1.0, num_probe_heads=3, max_sel_q=37,
                       max_spans=40)
    b8 = W.fp8_cache_variant(b, 561, k_std=1.0, v_std=1.0)
    got, want = _check(b8)
    assert want.abs().max() > 0.05
    few = W.random_batch(570 + d, [300, 150, 700], [45, 150, 1], 8, 2, d, torch.bfloat16, num_probe_heads=4, max_sel_q=5,
                         max_spans=6)
    few8 = W.fp8_cache_variant(few, 571).to(DEV)
    call = binding.call_from_batch(few8)
    call.launch()
    wide = binding.hook_span_mass_batch(few8)
    torch.cuda.synchronize()
    assert (call.mass - wide).abs().max().item() <= 2e-5
