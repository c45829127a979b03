"""Parity of the HIP library against the CPU oracle, through the C ABI (needs an MI355X)."""
import pytest
import torch

from paper_2603_06588_amd import workloads as W
import oracle
from helpers import MASS_ATOL as MASS_TOL, bits, compare_with_oracle, run_hip

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _check(b_cpu, rows=None, label=None, batch_kind=0):
    """batch_kind: the hint bench.py passes for this workload (the full-size cases are checked in the
    launch configuration that is timed)."""
    print(f"[case] {label or b_cpu.name} seqs={b_cpu.num_seqs} total_q={b_cpu.total_q}", flush=True)
    b = b_cpu.to(DEV)
    from paper_2603_06588_amd import binding
    # outputs start as NaN: a row or a mass entry that no work item writes cannot pass
    out = torch.full_like(b.q, float("nan"))
    mass = torch.full((b.num_seqs, b.num_probe_heads, b.max_sel_q, b.max_spans), float("nan"), dtype=torch.float32,
                      device=DEV)
    call = binding.call_from_batch(b, batch_kind=batch_kind, out=out, mass=mass)
    call.launch()
    torch.cuda.synchronize()
    assert call.device_status() == 0
    written = torch.isfinite(out.float()).all(dim=2).all(dim=1).cpu()
    from helpers import valid_rows
    assert bool((written == valid_rows(b_cpu)).all()), f"{label}: rows of out written != rows of valid sequences"
    res = compare_with_oracle(b_cpu, out, mass, rows=rows, label=label or b_cpu.name)
    print(f"       {res}", flush=True)
    return b, out, mass


# ---- small element-by-element cases: several tiles, ragged tails, both paths ----

SMALL = [
    # seed, seq_lens, q_lens, Hq, Hkv, d, std
    (101, [200], [200], 8, 2, 128, 1.0),                       # prefill, 4 tiles, G=4
    (102, [77, 130, 65, 64], [77, 130, 65, 64], 8, 2, 128, 1.0),  # ragged, tile-edge lengths
    (103, [300, 150], [45, 150], 8, 2, 128, 1.0),               # chunk on prior context
    (104, [500, 33, 257, 1025], [1, 1, 1, 1], 8, 2, 128, 1.0),  # decode, ragged contexts
    (105, [700, 90, 1, 260], [1, 90, 1, 3], 8, 2, 128, 1.0),    # mixed decode + prefill + tiny chunk
    (106, [190, 64], [190, 64], 8, 1, 128, 1.0),                # G=8
    (107, [150, 40], [150, 40], 6, 2, 128, 1.0),                # G=3 -> one head per wave
    (108, [150, 40], [150, 40], 4, 2, 128, 1.0),                # G=2
    (109, [140, 70], [140, 70], 4, 4, 128, 1.0),                # G=1
    (110, [210, 90, 300], [210, 1, 1], 8, 2, 64, 1.0),          # d=64, both paths
    (111, [129, 512], [129, 1], 16, 2, 128, 0.09),              # near-uniform attention
    (112, [40, 0, 25], [40, 0, 25], 8, 2, 128, 1.0),            # empty sequence in the middle
    (113, [2100], [1], 8, 8, 128, 1.0),                         # long single decode, G=1
    (114, [330, 330], [1, 1], 6, 2, 64, 1.0),                   # decode, G=3, d=64
]


@pytest.mark.parametrize("seed,lens,qlens,Hq,Hkv,d,std", SMALL)
def test_small_batches(seed, lens, qlens, Hq, Hkv, d, std):
    b = W.random_batch(seed, lens, qlens, Hq, Hkv, d, torch.bfloat16, std=std, num_probe_heads=min(5, Hq),
                       max_sel_q=6, max_spans=3)
    _check(b, label=f"small_{seed}")


def test_many_spans_and_rows():
    b = W.random_batch(120, [260, 100], [260, 100], 8, 2, 128, torch.bfloat16, num_probe_heads=8, max_sel_q=70,
                       max_spans=8)
    b.query_sel[0, 0], b.query_sel[0, 1] = 180, 250   # spans two row blocks and a tile edge
    _check(b, label="many_spans")


def test_all_rows_selected_beyond_4096():
    """Every row of a 4500-token prompt selected (the all-tokens query mode on a long prompt).  The
    oracle checks output and masses on a sample of rows; a span over the whole context pins the
    other rows (its mass is 1 at every row)."""
    L = 4500
    b = W.random_batch(125, [L, 300], [L, 300], 4, 2, 128, torch.bfloat16, num_probe_heads=2, max_sel_q=L,
                       max_spans=2)
    b.query_sel[0, 0], b.query_sel[0, 1] = 0, L
    b.key_spans[0, 1, 0], b.key_spans[0, 1, 1] = 0, L
    rows = sorted(set(list(range(0, 40)) + list(range(4080, 4120)) + list(range(L - 20, L + 300)) +
                      torch.randint(0, L, (64,), generator=torch.Generator().manual_seed(5)).tolist()))
    print(f"[case] all_rows_4500 sampled rows={len(rows)}", flush=True)
    out, mass = run_hip(b.to(DEV))
    assert mass.shape == (2, 2, L, 2)
    ref_out, ref_mass = oracle.attn_probe_batch(b, rows=rows)
    idx = torch.tensor(rows)
    err = (out.cpu().double()[idx] - ref_out[idx]).abs().max().item()
    assert err <= 2e-2 and err <= 2e-2 * ref_out[idx].abs().max().item()
    got = mass.cpu().double()
    long_rows = torch.tensor([t for t in rows if t < L])
    assert (got[0][:, long_rows] - ref_mass[0][:, long_rows]).abs().max().item() <= MASS_TOL
    assert (got[1] - ref_mass[1]).abs().max().item() <= MASS_TOL          # all 300 rows of the short one
    assert (got[0, :, :, 1] - 1.0).abs().max().item() <= MASS_TOL
    assert got.min().item() >= 0.0 and got.max().item() <= 1.0 + MASS_TOL
    # the separate span pass accepts the same selection and agrees with the attention kernels
    from paper_2603_06588_amd import binding
    wide = binding.hook_span_mass_batch(b.to(DEV))
    torch.cuda.synchronize()
    assert (wide.cpu().double() - got).abs().max().item() <= MASS_TOL


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 64)])
def test_query_sel_reaching_outside_the_chunk(dtype, d):
    """Row ranges that begin before the chunk or end after it, on single-row sequences, query chunks
    and the span pass: a row keeps slot t - begin, everything else stays zero (the oracle's rule)."""
    from paper_2603_06588_amd import binding
    lens, qlens = [500, 300, 64, 130, 90, 77], [1, 1, 64, 130, 1, 1]
    if dtype == torch.float32:
        lens, qlens = [90, 60, 33, 70, 20, 41], [1, 1, 33, 70, 1, 1]
    b = W.random_batch(126, lens, qlens, 8, 2, d, dtype, num_probe_heads=5, max_sel_q=6, max_spans=3)
    n2, n3 = qlens[2], qlens[3]
    sel = [[-2, 1], [-5, 3], [-3, 2], [n3 - 2, n3 + 9], [-6, 1], [1, 4]]
    # seq 0: slot 2; seq 1: slot 5; seq 2: rows 0, 1 in slots 3, 4; seq 3: the last two rows in slots 0, 1;
    # seq 4: the row would need slot 6 of 6: dropped; seq 5: a range past the only row: nothing
    b.query_sel[:] = torch.tensor(sel, dtype=torch.int32)
    _, _, mass = _check(b, label=f"query_sel_outside_{dtype}_{d}")
    got = mass.cpu()
    assert (got[0, :, 2] != 0).any() and (got[0, :, :2] == 0).all() and (got[0, :, 3:] == 0).all()
    assert (got[1, :, 5] != 0).any() and (got[1, :, :5] == 0).all()
    assert (got[2, :, :3] == 0).all() and (got[2, :, 5:] == 0).all()
    assert (got[3, :, 2:] == 0).all()
    assert (got[4] == 0).all() and (got[5] == 0).all()
    assert n2 > 2
    # the reductions count exactly the slots that hold a row
    from oracle.reduce import SPAN_MEAN, reduce_mass
    _, ref_mass = oracle.attn_probe_batch(b)
    want = reduce_mass(ref_mass.numpy(), SPAN_MEAN, 0, 1, b.query_sel.tolist(), b.cu_q_lens.tolist())
    bd = b.to(DEV)
    scores = binding.hook_reduce_mass(mass, SPAN_MEAN, 0, 1, bd.query_sel, bd.cu_q_lens)
    torch.cuda.synchronize()
    assert (scores.cpu().double() - torch.from_numpy(want)).abs().max().item() <= 2e-3
    if dtype == torch.bfloat16:
        wide = binding.hook_span_mass_batch(bd)
        torch.cuda.synchronize()
        assert (wide.cpu().double() - got.double()).abs().max().item() <= MASS_TOL


def test_fp32_small():
    b = W.random_batch(130, [100, 37, 64], [100, 5, 1], 8, 2, 64, torch.float32, num_probe_heads=4, max_sel_q=4,
                       max_spans=2)
    _check(b, label="fp32_small")
    b = W.random_batch(131, [70, 20], [70, 1], 4, 2, 128, torch.float32, num_probe_heads=4, max_sel_q=4, max_spans=2)
    _check(b, label="fp32_small_d128")


# ---- invariants that must hold bit for bit ----

@pytest.mark.parametrize("lens,qlens", [([333, 150], [333, 150]), ([900, 450, 64], [1, 1, 1]), ([400, 200], [1, 200])])
def test_paging_permutation_is_bit_exact(lens, qlens):
    kw = dict(num_q_heads=8, num_kv_heads=2, head_dim=128, dtype=torch.bfloat16, num_probe_heads=4)
    shuf = W.random_batch(140, lens, qlens, shuffle=True, poison=True, **kw)
    ident = W.random_batch(140, lens, qlens, shuffle=False, poison=False, **kw)
    ident.q = shuf.q.clone()
    ident.query_sel, ident.key_spans, ident.probe_heads = shuf.query_sel, shuf.key_spans, shuf.probe_heads
    for i, L in enumerate(lens):
        for jb in range((L + 15) // 16):
            ident.k_cache[int(ident.block_table[i, jb])] = shuf.k_cache[int(shuf.block_table[i, jb])]
            ident.v_cache[int(ident.block_table[i, jb])] = shuf.v_cache[int(shuf.block_table[i, jb])]
    o1, m1 = run_hip(shuf.to(DEV))
    o2, m2 = run_hip(ident.to(DEV))
    assert torch.equal(bits(o1), bits(o2))
    assert torch.equal(bits(m1), bits(m2))
    assert torch.isfinite(o1.float()).all()


def test_two_runs_bit_identical_and_probe_does_not_change_out():
    b_cpu = W.random_batch(150, [520, 300, 800, 64], [520, 1, 1, 64], 8, 2, 128, torch.bfloat16, num_probe_heads=6,
                           max_sel_q=8, max_spans=4)
    b = b_cpu.to(DEV)
    o1, m1 = run_hip(b)
    o2, m2 = run_hip(b)
    assert torch.equal(bits(o1), bits(o2)) and torch.equal(bits(m1), bits(m2))
    o3, m3 = run_hip(b, probe=False)
    assert torch.equal(bits(o1), bits(o3))
    assert m3.numel() == 0


def test_mass_is_fully_written():
    from paper_2603_06588_amd import binding
    b_cpu = W.random_batch(151, [100, 50, 10], [100, 1, 0], 8, 2, 128, torch.bfloat16, num_probe_heads=3, max_sel_q=5,
                           max_spans=3)
    b = b_cpu.to(DEV)
    mass = torch.full((3, 3, 5, 3), float("nan"), dtype=torch.float32, device=DEV)
    call = binding.call_from_batch(b, mass=mass)
    call.launch()
    torch.cuda.synchronize()
    assert torch.isfinite(mass).all()
    compare_with_oracle(b_cpu, call.out, mass, label="mass_written")
    assert call.device_status() == 0


def test_uniform_attention_closed_form_on_gpu():
    b_cpu = W.random_batch(152, [300, 700], [300, 1], 8, 2, 128, torch.bfloat16, num_probe_heads=8, max_sel_q=4,
                           max_spans=3, wild_spans=False)
    b_cpu.q.zero_()
    b = b_cpu.to(DEV)
    out, mass = run_hip(b)
    qs, ks = b_cpu.query_sel.tolist(), b_cpu.key_spans.tolist()
    for i, (L, n) in enumerate([(300, 300), (700, 1)]):
        for tt in range(qs[i][1] - qs[i][0]):
            pos = L - n + qs[i][0] + tt
            for r in range(3):
                a, e = ks[i][r]
                want = max(0, min(e, pos + 1) - max(a, 0)) / (pos + 1)
                assert (mass[i, :, tt, r].cpu() - want).abs().max() < 1e-5


# ---- the named workloads ----

def test_c1_tiny_prefill_fp32():
    b, s = W.c1_tiny_prefill()
    _check(b, label="c1")


@pytest.mark.parametrize("peaked", [False, True])
def test_c2_c3_c5_shrunk(peaked):
    _check(W.c2_prefill_8b(peaked=peaked, shrink=4), label=f"c2_shrink4_peaked{peaked}")
    _check(W.c3_decode_8b(peaked=peaked, shrink=8), label=f"c3_shrink8_peaked{peaked}")
    b5, _ = W.c5_mixed(peaked=peaked, shrink=8)
    _check(b5, label=f"c5_shrink8_peaked{peaked}")
    b5p, _ = W.c5_mixed(peaked=peaked, shrink=8, prior_context=True)
    _check(b5p, label=f"c5_prior_shrink8_peaked{peaked}")
    _check(W.c4_long_prefill_70b(peaked=peaked, shrink=16), label=f"c4_shrink16_peaked{peaked}")


def _sample_rows(b, per_seq: int, seed: int):
    """Probed rows plus tile-boundary and seeded-random rows of every sequence."""
    gen = torch.Generator().manual_seed(seed)
    cu = b.cu_q_lens.tolist()
    qs = b.query_sel.tolist()
    rows = set()
    for i in range(b.num_seqs):
        n = cu[i + 1] - cu[i]
        if n == 0:
            continue
        for t in range(max(qs[i][0], 0), min(qs[i][1], n)):
            rows.add(cu[i] + t)
        fixed = [0, 1, 31, 32, 63, 64, 65, 127, 128, n // 2, n - 65, n - 64, n - 33, n - 32, n - 1]
        rnd = torch.randint(0, n, (per_seq,), generator=gen).tolist()
        for t in fixed + rnd:
            if 0 <= t < n:
                rows.add(cu[i] + t)
    return sorted(rows)


def test_c2_full_size_every_row():
    b = W.c2_prefill_8b()
    _check(b, label="c2_full", batch_kind=1)


def test_c2_full_size_peaked_every_row():
    b = W.c2_prefill_8b(peaked=True)
    _check(b, label="c2_full_peaked")


def test_c3_full_size():
    b = W.c3_decode_8b(device="cpu")
    _check(b, label="c3_full", batch_kind=2)


def _stratified_rows(b, block: int, seed: int):
    """One seeded-random row out of every `block` consecutive rows (every work item of the long
    prefill is hit), on top of the probed and tile-boundary rows."""
    gen = torch.Generator().manual_seed(seed)
    rows = set(_sample_rows(b, 0, seed))
    for r0 in range(0, b.total_q, block):
        rows.add(r0 + int(torch.randint(0, min(block, b.total_q - r0), (1,), generator=gen)))
    return sorted(rows)


@pytest.mark.parametrize("peaked", [False, True])
def test_c4_full_size_stratified_rows(peaked):
    b = W.c4_long_prefill_70b(peaked=peaked)
    _check(b, rows=_stratified_rows(b, 32, 3), label=f"c4_full_peaked{peaked}", batch_kind=1)


def test_c5_full_size_every_row():
    b, s = W.c5_mixed()
    _check(b, label="c5_full")


# ---- malformed device-side contents must be made safe, flagged and never fault ----

def test_bad_lengths_are_flagged_and_skipped():
    from paper_2603_06588_amd import binding
    b_cpu = W.random_batch(160, [200, 300, 150, 90], [200, 1, 150, 1], 8, 2, 128, torch.bfloat16, num_probe_heads=3,
                           max_sel_q=4, max_spans=2)
    ref = b_cpu.to(DEV)
    out_ok, mass_ok = run_hip(ref)
    bad = b_cpu.to(DEV)
    bad.seq_lens = bad.seq_lens.clone()
    bad.seq_lens[2] = 100                      # n_i (150) > L_i: sequence 2 is skipped
    bad.seq_lens[3] = 16 * b_cpu.max_blocks_per_seq + 500   # beyond the table: clamped
    bad.block_table = bad.block_table.clone()
    bad.block_table[3] = torch.where(bad.block_table[3] > b_cpu.num_blocks, torch.zeros_like(bad.block_table[3]),
                                     bad.block_table[3])
    out = torch.full_like(out_ok, 7.0)
    call = binding.call_from_batch(bad, out=out)
    call.launch()
    torch.cuda.synchronize()
    bits_ = call.device_status()
    assert bits_ & 1 and bits_ & 2
    cu = b_cpu.cu_q_lens.tolist()
    # untouched rows of the skipped sequence, bit-identical rows of the valid ones
    assert (out[cu[2]:cu[3]] == 7.0).all()
    assert torch.equal(bits(out[cu[0]:cu[2]]), bits(out_ok[cu[0]:cu[2]]))
    # (sequence 3 attends to whatever the clamped table rows point at: its values are undefined,
    # the point is that the call completed without touching memory outside the cache)
    assert torch.equal(bits(call.mass[:2]), bits(mass_ok[:2]))
    assert (call.mass[2] == 0).all()


def test_garbage_block_ids_do_not_fault():
    b_cpu = W.random_batch(161, [260, 700], [260, 1], 8, 2, 128, torch.bfloat16, num_probe_heads=2, poison=False)
    b = b_cpu.to(DEV)
    b.block_table = torch.full_like(b.block_table, 0x7FFFFFF0)
    b.block_table[0, 0] = -5
    out, mass = run_hip(b)      # values are meaningless, but every access stays inside the cache
    assert out.shape == b.q.shape


# ---- the call is a fixed launch sequence: it can be replayed from a HIP graph ----

def test_hip_graph_replay_matches_eager():
    from paper_2603_06588_amd import binding
    b_cpu = W.random_batch(170, [400, 900, 128, 333], [400, 1, 128, 1], 8, 2, 128, torch.bfloat16, num_probe_heads=4,
                           max_sel_q=4, max_spans=2)
    b = b_cpu.to(DEV)
    eager_out, eager_mass = run_hip(b)
    call = binding.call_from_batch(b)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        call.launch(s)              # warm-up on the side stream (sets kernel attributes)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        call.launch(torch.cuda.current_stream())
    for rep in range(3):
        call.out.fill_(float("nan"))
        call.mass.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(bits(call.out), bits(eager_out)), rep
        assert torch.equal(bits(call.mass), bits(eager_mass)), rep
        # eager work between replays
        again_out, _ = run_hip(b)
        assert torch.equal(bits(again_out), bits(eager_out))


def test_many_prefill_sequences_overflow_the_planner_queue():
    # more prefill sequences than the planner's queue holds: the overflow path must give the same result
    nseq = 1100
    lens = [2 + (i % 5) for i in range(nseq)]
    b = W.random_batch(180, lens, lens, 4, 2, 128, torch.bfloat16, num_probe_heads=2, max_sel_q=2, max_spans=1)
    _check(b, label="planner_overflow")


def test_many_decode_sequences_take_several_planner_trips():
    # more single-row sequences than the planner has threads, ragged contexts from one key to several
    # chunks, two query chunks and an empty sequence in between
    lens, qlens = [], []
    for i in range(2300):
        L = 1 + (i * 37) % 700
        lens.append(L)
        qlens.append(1)
    lens[5], qlens[5] = 90, 90
    lens[1500], qlens[1500] = 300, 40
    lens[2000], qlens[2000] = 0, 0
    b = W.random_batch(181, lens, qlens, 4, 2, 128, torch.bfloat16, num_probe_heads=2, max_sel_q=1, max_spans=2)
    _check(b, label="planner_many_decodes")


def test_validate_reports_what_the_kernels_only_make_safe():
    """hook_attn_probe_validate on a clean batch and on one corruption at a time."""
    from paper_2603_06588_amd import binding as B
    def bits_of(mutate=None, **kw):
        b = W.random_batch(195, [300, 77, 150, 40], [300, 1, 90, 0], 8, 2, 128, torch.bfloat16, num_probe_heads=3,
                           max_sel_q=4, max_spans=2, poison=False).to(DEV)
        if mutate:
            mutate(b)
        return B.call_from_batch(b, **kw).validate()
    assert bits_of() == 0
    def rows_exceed(b): b.seq_lens[2] = 50                      # n = 90 > L = 50
    assert bits_of(rows_exceed) & B.BAD_ROWS_EXCEED_CONTEXT
    def too_long(b): b.seq_lens[0] = b.block_table.shape[1] * 16 + 1
    assert bits_of(too_long) & B.BAD_CONTEXT_TOO_LONG
    def negative(b): b.seq_lens[1] = -3
    assert bits_of(negative) & B.BAD_LENGTH
    def bad_prefix(b): b.cu_q_lens[4] = b.total_q - 1           # last entry must equal total_q
    assert bits_of(bad_prefix) & B.BAD_LENGTH
    def bad_block(b): b.block_table[0, 3] = 10 ** 6
    assert bits_of(bad_block) == B.BAD_BLOCK_ID
    def dead_entry(b): b.block_table[1, b.block_table.shape[1] - 1] = -5   # past the live context: not read
    assert bits_of(dead_entry) == 0
    def unsorted(b): b.probe_heads[1] = b.probe_heads[0]
    assert bits_of(unsorted) == B.BAD_PROBE_HEADS
    def clipped(b): b.query_sel[0, 0], b.query_sel[0, 1] = 298, 302          # reaches past n = 300: clipped
    assert bits_of(clipped) == 0
    def before(b): b.query_sel[1, 0], b.query_sel[1, 1] = -2, 1              # begins before the chunk: clipped
    assert bits_of(before) == 0
    def sel(b): b.query_sel[0, 0], b.query_sel[0, 1] = 290, 300              # 10 rows into 4 slots
    assert bits_of(sel) == B.BAD_QUERY_SEL
    def sel_neg(b): b.query_sel[1, 0], b.query_sel[1, 1] = -4, 1             # the single row would need slot 4
    assert bits_of(sel_neg) == B.BAD_QUERY_SEL
    assert bits_of(batch_kind=B.BATCH_PREFILL_ONLY) == B.BAD_BATCH_KIND      # sequence 1 is a single row
    assert bits_of(batch_kind=B.BATCH_DECODE_ONLY) == B.BAD_BATCH_KIND


def test_plan_reuse_across_layers():
    """One plan per model step: later calls on the same batch (other q / caches / probe arguments)
    reuse the work lists in the workspace, skip the planner and give the same bits as fresh calls;
    entries of `mass` that no selected row maps to are left as they were."""
    from paper_2603_06588_amd import binding as B
    lens, qlens = [300, 77, 1500, 150, 40, 9], [300, 1, 1, 90, 0, 9]
    layer0 = W.random_batch(196, lens, qlens, 8, 2, 128, torch.bfloat16, num_probe_heads=3, max_sel_q=4, max_spans=2).to(DEV)
    layer1 = W.random_batch(197, lens, qlens, 8, 2, 128, torch.bfloat16, num_probe_heads=5, max_sel_q=4, max_spans=2).to(DEV)
    fresh0 = B.call_from_batch(layer0)
    fresh0.launch()
    want1_out, want1_mass = run_hip(layer1)
    # the second layer shares layer 0's workspace and block table layout (same lengths), not its tensors
    marker = 123.25
    mass1 = torch.full_like(want1_mass, marker)
    reuse1 = B.call_from_batch(layer1, workspace=fresh0.workspace, mass=mass1, plan_mode=B.PLAN_REUSE)
    reuse1.out.fill_(float("nan"))
    from paper_2603_06588_amd import benchlib
    times = benchlib.launch_timed(reuse1)
    torch.cuda.synchronize()
    assert times[0] == 0.0                                     # no planner
    assert torch.equal(bits(reuse1.out[:300]), bits(want1_out[:300]))
    valid_rows = torch.ones(layer1.total_q, dtype=torch.bool)
    assert torch.equal(bits(reuse1.out[valid_rows]), bits(want1_out[valid_rows]))
    written = mass1 != marker
    assert torch.equal(bits(mass1[written]), bits(want1_mass[written]))
    assert (want1_mass[~written] == 0).all()                   # what was left alone is what a fresh call zero-fills
    assert written.any() and (~written).any()
    assert reuse1.device_status() == 0


def test_batch_kind_hint():
    """A correct hint changes nothing but the launches (and, for few single rows, the split of the contexts); a wrong one drops the contradicting
    sequences (rows untouched, mass zero) and sets bit 3 of the status word."""
    from paper_2603_06588_amd import binding
    pre = W.random_batch(190, [300, 77, 150], [300, 2, 90], 8, 2, 128, torch.bfloat16, num_probe_heads=3, max_sel_q=3,
                         max_spans=2).to(DEV)
    dec = W.random_batch(191, [300, 77, 1500], [1, 1, 1], 8, 2, 128, torch.bfloat16, num_probe_heads=3, max_sel_q=1,
                         max_spans=2).to(DEV)
    for b, kind in ((pre, binding.BATCH_PREFILL_ONLY), (dec, binding.BATCH_DECODE_ONLY)):
        ref_out, ref_mass = run_hip(b)
        call = binding.call_from_batch(b, batch_kind=kind)
        call.out.fill_(float("nan"))
        call.launch()
        torch.cuda.synchronize()
        if kind == binding.BATCH_PREFILL_ONLY:
            assert torch.equal(bits(call.out), bits(ref_out)) and torch.equal(bits(call.mass), bits(ref_mass))
        else:
            # a small batch of single rows cuts its contexts into equal parts instead of planned chunks:
            # the same sums in another order
            assert torch.allclose(call.out.float(), ref_out.float(), atol=2e-2, rtol=2e-2)
            assert torch.allclose(call.mass, ref_mass, atol=1e-3)
        assert call.device_status() == 0
        from paper_2603_06588_amd import benchlib
        ms = benchlib.launch_timed(call)
        assert ms[1 if kind == binding.BATCH_DECODE_ONLY else 2] == 0.0     # the other side was not launched
    mixed = W.random_batch(192, [300, 77, 150, 40], [300, 1, 90, 1], 8, 2, 128, torch.bfloat16, num_probe_heads=3,
                           max_sel_q=3, max_spans=2).to(DEV)
    ref_out, ref_mass = run_hip(mixed)
    call = binding.call_from_batch(mixed, batch_kind=binding.BATCH_PREFILL_ONLY)
    call.out.fill_(7.0)
    call.launch()
    torch.cuda.synchronize()
    assert call.device_status() & 8
    cu = mixed.cu_q_lens.tolist()
    for i, n in enumerate([300, 1, 90, 1]):
        rows = slice(cu[i], cu[i + 1])
        if n == 1:
            assert (call.out[rows] == 7.0).all() and (call.mass[i] == 0).all()
        else:
            assert torch.equal(bits(call.out[rows]), bits(ref_out[rows]))
            assert torch.equal(bits(call.mass[i]), bits(ref_mass[i]))


@pytest.mark.parametrize("group", [0, 1, 2, 3])
def test_random_valid_batches(group):
    """Seeded random batches (head geometry, head_dim, dtype, ragged lengths, chunk / single-row / empty
    sequences, probe set) through the attention entry point and the span pass, against the oracle."""
    import random
    from paper_2603_06588_amd import binding
    rng = random.Random(9000 + group)
    for it in range(12):
        G, Hkv = rng.choice([1, 2, 3, 4, 8]), rng.choice([1, 2, 4])
        d = rng.choice([128, 128, 64])
        dtype = torch.bfloat16 if rng.random() < 0.85 else torch.float32
        if dtype == torch.float32:
            lens = [rng.randint(1, 90) for _ in range(rng.randint(1, 3))]
        else:
            lens = [rng.choice([rng.randint(1, 40), rng.randint(41, 300), rng.randint(300, 1200)])
                    for _ in range(rng.randint(1, 6))]
        qlens = []
        for L in lens:
            r = rng.random()
            qlens.append(1 if r < 0.35 else L if r < 0.7 else 0 if r < 0.78 else rng.randint(1, L))
        if sum(qlens) == 0:
            qlens[0] = 1
        b = W.random_batch(9100 + 100 * group + it, lens, qlens, G * Hkv, Hkv, d, dtype, std=rng.choice([1.0, 1.0, 0.09]),
                           num_probe_heads=rng.randint(1, G * Hkv), max_sel_q=rng.choice([1, 2, 5, 33]),
                           max_spans=rng.randint(1, 8))
        label = f"random g{group} #{it} lens={lens} q={qlens} Hq={G * Hkv} Hkv={Hkv} d={d} {dtype}"
        _, _, mass = _check(b, label=label)
        if dtype == torch.bfloat16:
            wide = binding.hook_span_mass_batch(b.to(DEV))
            torch.cuda.synchronize()
            assert (wide.cpu().double() - mass.cpu().double()).abs().max().item() <= MASS_TOL, label
