"""Small batches of single rows plan themselves: every sequence is cut into equally many parts by the
workgroups, and no planning launch runs.  These cases pin that path against the CPU oracle through the
C ABI (needs an MI355X); each has at most 512 (sequence, kv head, head group) triples, which is what
selects it."""
import pytest
import torch

from paper_2603_06588_amd import binding, workloads as W
from helpers import bits, compare_with_oracle, run_hip

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(b_cpu, probe=True, sentinel=float("nan"), **kw):
    b = b_cpu.to(DEV)
    out = torch.full_like(b.q, sentinel)
    mass = torch.full((b.num_seqs, b.num_probe_heads, b.max_sel_q, b.max_spans), float("nan"), dtype=torch.float32,
                      device=DEV)
    call = binding.call_from_batch(b, probe=probe, batch_kind=binding.BATCH_DECODE_ONLY, out=out,
                                   mass=mass if probe else None, **kw)
    call.workspace.fill_(0xFF)
    call.launch()
    torch.cuda.synchronize()
    # the first words of the workspace are [chunk items, single-row items, chunk length, status]:
    # all zero here, because no planner ran and the workgroups wrote the status themselves
    hdr = call.workspace[:16].view(torch.int32).tolist()
    assert hdr[:3] == [0, 0, 0], f"the batch did not take the self-planned path: {hdr}"
    return call


CASES = [
    # seed, context lengths, Hq, Hkv, d, std
    (1201, [500, 33, 257, 1025, 1, 15, 16, 17, 255, 256, 2100, 64, 48, 700, 90, 260], 8, 2, 128, 1.0),  # G = 4
    (1202, [2100, 1, 300, 31], 8, 8, 128, 1.0),                                   # G = 1
    (1203, [330, 330, 17, 1000, 5, 129], 6, 2, 64, 1.0),                           # G = 3 (one head per group), d = 64
    (1204, [700, 90, 1, 260] * 4, 16, 2, 128, 0.09),                               # G = 8, near-uniform attention
    (1205, [64, 48, 16, 15, 1, 400, 33, 32] * 2 + [1500] * 4, 4, 2, 64, 1.0),      # G = 2, d = 64
    (1206, [3000, 2500, 40, 4100, 777], 32, 8, 128, 0.5),                          # the 8B head geometry
    (1207, [100 + 37 * i for i in range(32)], 32, 8, 128, 1.0),                    # 256 (sequence, kv head) pairs: few parts each
]


@pytest.mark.parametrize("seed,lens,Hq,Hkv,d,std", CASES)
def test_self_planned_decode_matches_the_oracle(seed, lens, Hq, Hkv, d, std):
    print(f"[case] self-planned decode seed={seed} seqs={len(lens)} Hq={Hq} Hkv={Hkv} d={d}", flush=True)
    b = W.random_batch(seed, lens, [1] * len(lens), Hq, Hkv, d, torch.bfloat16, std=std, num_probe_heads=min(5, Hq),
                       max_sel_q=2, max_spans=3)
    b.query_sel[:, 0], b.query_sel[:, 1] = 0, 1
    b.query_sel[1, 0], b.query_sel[1, 1] = -1, 1         # the row lands in slot 1, slot 0 stays zero
    b.query_sel[2, 0], b.query_sel[2, 1] = 1, 2          # the row is not selected
    call = _run(b)
    assert call.device_status() == 0
    assert torch.isfinite(call.out.float()).all()
    res = compare_with_oracle(b, call.out, call.mass, label=f"selfplan_{seed}")
    print(res, flush=True)
    assert (call.mass[1, :, 0] == 0).all() and (call.mass[2] == 0).all()
    # switching the probe off changes no bit of out; a second run changes nothing either
    c2 = _run(b, probe=False)
    assert torch.equal(bits(call.out), bits(c2.out))
    c3 = _run(b)
    assert torch.equal(bits(call.out), bits(c3.out)) and torch.equal(bits(call.mass), bits(c3.mass))


def test_self_planned_decode_fp8_cache():
    lens = [500, 33, 257, 1025, 1, 15, 16, 17, 3000, 2500]
    b = W.random_batch(1210, lens, [1] * len(lens), 32, 8, 128, torch.bfloat16, num_probe_heads=5, max_sel_q=1, max_spans=3)
    b8 = W.fp8_cache_variant(b, 1211, k_std=0.5, v_std=1.0)
    call = _run(b8)
    assert call.device_status() == 0
    print(compare_with_oracle(b8, call.out, call.mass, label="selfplan_kv8"), flush=True)


def test_self_planned_decode_skips_and_flags_what_the_planner_would():
    """Empty sequences, a row block in a batch promised to hold single rows, a length beyond the table
    and a negative length: the same status bits and the same untouched rows as on the planned path."""
    lens = [300, 77, 150, 40, 500, 90, 200, 64] * 2
    qlens = [1] * 16
    qlens[3], qlens[5] = 0, 3            # an empty sequence, a row block (contradicts the hint)
    b_cpu = W.random_batch(1220, lens, qlens, 8, 2, 128, torch.bfloat16, num_probe_heads=3, max_sel_q=1, max_spans=2)
    b_cpu.query_sel[:, 0], b_cpu.query_sel[:, 1] = 0, 1
    bad = b_cpu.to("cpu")
    bad.seq_lens = bad.seq_lens.clone()
    bad.seq_lens[7] = -4                                      # negative: skipped
    bad.seq_lens[9] = 16 * b_cpu.max_blocks_per_seq + 500     # beyond the table: clamped
    bad.block_table = bad.block_table.clone()
    bad.block_table[9] = torch.where(bad.block_table[9] > b_cpu.num_blocks, torch.zeros_like(bad.block_table[9]),
                                     bad.block_table[9])
    call = _run(bad, sentinel=7.0)
    st = call.device_status()
    assert st == (2 | 4 | 8), st
    # the planned path (no hint) on the same, valid part of the batch
    good = b_cpu.to(DEV)
    ref_out, ref_mass = run_hip(good)
    cu = b_cpu.cu_q_lens.tolist()
    for i in range(16):
        rows = slice(cu[i], cu[i + 1])
        if i in (3, 5, 7):
            assert (call.out[rows] == 7.0).all() and (call.mass[i] == 0).all()
        elif i != 9:
            assert torch.allclose(call.out[rows].float(), ref_out[rows].float(), atol=2e-2, rtol=2e-2)
            assert torch.allclose(call.mass[i], ref_mass[i], atol=2e-3)


def test_self_planned_decode_with_new_rows_written_in_the_call():
    """k_new / v_new: the cache rows of the new tokens are written before the workgroups read them."""
    lens = [500, 33, 257, 1025, 1, 16, 17, 700]
    b_cpu = W.random_batch(1230, lens, [1] * len(lens), 32, 8, 128, torch.bfloat16, num_probe_heads=4, max_sel_q=1,
                           max_spans=2)
    b_cpu.query_sel[:, 0], b_cpu.query_sel[:, 1] = 0, 1
    ref = _run(b_cpu)
    # wipe the last key/value row of every sequence from the cache and hand it over as k_new / v_new
    b = b_cpu.to(DEV)
    k_new = torch.empty(b.total_q, 8, 128, dtype=torch.bfloat16, device=DEV)
    v_new = torch.empty_like(k_new)
    for i, L in enumerate(lens):
        blk, off = int(b.block_table[i, (L - 1) // 16]), (L - 1) % 16
        k_new[i], v_new[i] = b.k_cache[blk, :, off], b.v_cache[blk, :, off]
        b.k_cache[blk, :, off] = float("nan")
        b.v_cache[blk, :, off] = float("nan")
    out = torch.full_like(b.q, float("nan"))
    call = binding.call_from_batch(b, batch_kind=binding.BATCH_DECODE_ONLY, out=out, k_new=k_new, v_new=v_new)
    call.launch()
    torch.cuda.synchronize()
    assert torch.equal(bits(call.out), bits(ref.out)) and torch.equal(bits(call.mass), bits(ref.mass))


def test_self_planned_decode_reusing_call_writes_selected_entries_only():
    lens = [300, 77, 150, 40, 500, 90, 200, 64] * 2
    b_cpu = W.random_batch(1240, lens, [1] * 16, 8, 2, 128, torch.bfloat16, num_probe_heads=3, max_sel_q=2, max_spans=2)
    b_cpu.query_sel[:, 0], b_cpu.query_sel[:, 1] = 0, 1
    fresh = _run(b_cpu)
    b = b_cpu.to(DEV)
    mass = torch.full_like(fresh.mass, 5.0)
    call = binding.call_from_batch(b, batch_kind=binding.BATCH_DECODE_ONLY, plan_mode=binding.PLAN_REUSE, mass=mass,
                                   workspace=fresh.workspace)
    call.launch()
    torch.cuda.synchronize()
    assert torch.equal(bits(call.out), bits(fresh.out))
    assert torch.equal(bits(call.mass[:, :, 0]), bits(fresh.mass[:, :, 0]))
    assert (call.mass[:, :, 1] == 5.0).all()          # slot 1 holds no row: never written by a reusing call


@pytest.mark.parametrize("static_scratch", [False, True])
def test_self_planned_decode_replays_from_a_hip_graph(static_scratch):
    """The serving case this path is for: a captured decode step replayed several times, with eager work
    and synchronisations in between, on a caller workspace and on the library's own scratch array."""
    lens = [500, 33, 257, 1025, 1, 700, 90, 2100]
    b = W.random_batch(1250, lens, [1] * len(lens), 32, 8, 128, torch.bfloat16, num_probe_heads=4, max_sel_q=1,
                       max_spans=2)
    b.query_sel[:, 0], b.query_sel[:, 1] = 0, 1
    eager = _run(b)
    call = binding.call_from_batch(b.to(DEV), batch_kind=binding.BATCH_DECODE_ONLY)
    launch = call.launch_static if static_scratch else call.launch
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        launch(s)                       # warm-up on the side stream
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        launch(torch.cuda.current_stream())
    for rep in range(3):
        call.out.fill_(float("nan"))
        call.mass.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(bits(call.out), bits(eager.out)), rep
        assert torch.equal(bits(call.mass), bits(eager.mass)), rep
        again = _run(b)                 # eager work between the replays
        assert torch.equal(bits(again.out), bits(eager.out))


@pytest.mark.parametrize("group", [0, 1])
def test_random_decode_only_batches(group):
    """Seeded random single-row batches with the decode-only hint: head geometry, head_dim, number of
    sequences on both sides of the self-planning limit, empty sequences, both cache types, probe set and
    row selections (including ranges that begin before the row), against the oracle."""
    import random
    rng = random.Random(9500 + group)
    for it in range(10):
        G, Hkv = rng.choice([1, 2, 3, 4, 8]), rng.choice([1, 2, 4, 8])
        d = rng.choice([128, 128, 64])
        nseq = rng.choice([1, 3, 9, 40, 150])
        lens = [rng.choice([rng.randint(1, 40), rng.randint(41, 300), rng.randint(300, 2500)]) for _ in range(nseq)]
        qlens = [0 if rng.random() < 0.1 else 1 for _ in lens]
        if sum(qlens) == 0:
            qlens[0] = 1
        nq = rng.choice([1, 2, 4])
        b = W.random_batch(9600 + 100 * group + it, lens, qlens, G * Hkv, Hkv, d, torch.bfloat16,
                           std=rng.choice([1.0, 1.0, 0.09]), num_probe_heads=rng.randint(1, G * Hkv), max_sel_q=nq,
                           max_spans=rng.randint(1, 8))
        for i in range(nseq):
            begin = rng.choice([0, 0, 0, -1, 1, -(nq - 1)])
            b.query_sel[i, 0], b.query_sel[i, 1] = begin, begin + rng.randint(0, nq + 1)
        kv8 = rng.random() < 0.4
        if kv8:
            b = W.fp8_cache_variant(b, 9700 + it, k_std=rng.choice([1.0, 0.3]), v_std=1.0)
        label = f"random decode g{group} #{it} nseq={nseq} Hq={G * Hkv} Hkv={Hkv} d={d} kv8={kv8}"
        print(f"[case] {label}", flush=True)
        bd = b.to(DEV)
        out = torch.full_like(bd.q, float("nan"))
        mass = torch.full((b.num_seqs, b.num_probe_heads, b.max_sel_q, b.max_spans), float("nan"), dtype=torch.float32,
                          device=DEV)
        call = binding.call_from_batch(bd, batch_kind=binding.BATCH_DECODE_ONLY, out=out, mass=mass)
        call.launch()
        torch.cuda.synchronize()
        assert call.device_status() == 0, label
        from helpers import valid_rows
        written = torch.isfinite(out.float()).all(dim=2).all(dim=1).cpu()
        assert bool((written == valid_rows(b)).all()), label
        print("      ", compare_with_oracle(b, out, mass, label=label), flush=True)
