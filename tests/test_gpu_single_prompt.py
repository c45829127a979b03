"""One sequence of query rows on its own (the single-prompt case) plans itself inside the chunk kernel: no
planning launch.  Results must equal the planned path bit for bit (same work items, same code) and the
oracle within tolerance, and `mass` must be written entry by entry without a planner's zero-fill
(needs an MI355X)."""
import pytest
import torch

from paper_2603_06588_amd import binding, workloads as W
from helpers import bits, compare_with_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(b_cpu, kind, sentinel=float("nan"), **kw):
    b = b_cpu.to(DEV)
    out = torch.full_like(b.q, sentinel)
    mass = torch.full((b.num_seqs, b.num_probe_heads, b.max_sel_q, b.max_spans), float("nan"), dtype=torch.float32,
                      device=DEV)
    call = binding.call_from_batch(b, batch_kind=kind, out=out, mass=mass, **kw)
    call.workspace.fill_(0xFF)
    call.launch()
    torch.cuda.synchronize()
    return call


CASES = [
    # seed, L, n, Hq, Hkv, query_sel, label
    (1401, 2048, 2048, 32, 8, (2047, 2048), "a 2048-token prompt, last row"),
    (1402, 777, 777, 8, 2, (770, 777), "ragged length, last 7 rows"),
    (1403, 1500, 300, 8, 2, (-3, 2), "a chunk on prior context; the range begins before the chunk"),
    (1404, 333, 333, 6, 2, (330, 340), "G = 3 (one head per wave); the range reaches past the chunk"),
    (1405, 200, 200, 4, 2, (0, 0), "G = 2; nothing selected"),
    (1406, 190, 190, 4, 4, (100, 104), "G = 1; rows in the middle"),
    (1407, 65, 2, 16, 2, (0, 2), "two rows on prior context, G = 8"),
    (1408, 4100, 4100, 8, 2, (0, 4100), "all rows selected, more than 4096 slots"),
]


@pytest.mark.parametrize("seed,L,n,Hq,Hkv,sel,label", CASES)
def test_single_prompt_equals_planned_path_and_oracle(seed, L, n, Hq, Hkv, sel, label):
    print(f"[case] single prompt: {label}", flush=True)
    nq = max(4, min(sel[1] - sel[0], 4100)) if sel[1] > sel[0] else 4
    b = W.random_batch(seed, [L], [n], Hq, Hkv, 128, torch.bfloat16, num_probe_heads=min(5, Hq), max_sel_q=nq,
                       max_spans=3)
    b.query_sel[0, 0], b.query_sel[0, 1] = sel
    own = _run(b, binding.BATCH_PREFILL_ONLY)
    # the words a planner would have left: [row blocks, 0, 0, status]
    hdr = own.workspace[:16].view(torch.int32).tolist()
    assert hdr[1:4] == [0, 0, 0] and hdr[0] > 0, hdr
    planned = _run(b, binding.BATCH_MIXED)
    assert planned.workspace[:16].view(torch.int32).tolist()[0] == hdr[0]
    assert torch.equal(bits(own.out), bits(planned.out))
    assert torch.equal(bits(own.mass), bits(planned.mass))          # also: no entry left at the NaN it started with
    print("      ", compare_with_oracle(b, own.out, own.mass, label=label), flush=True)


def test_single_prompt_invalid_contents_are_flagged():
    b = W.random_batch(1410, [300], [300], 8, 2, 128, torch.bfloat16, num_probe_heads=3, max_sel_q=2, max_spans=2)

    def variant(L=None, n=None):
        v = b.to("cpu")
        v.seq_lens = v.seq_lens.clone()
        v.cu_q_lens = v.cu_q_lens.clone()
        if L is not None:
            v.seq_lens[0] = L
        if n is not None:
            v.cu_q_lens[1] = n
        return v

    for v, want in ((variant(L=100), 1), (variant(n=1), 8), (variant(L=-5), 4), (variant(n=0), 0)):
        call = _run(v, binding.BATCH_PREFILL_ONLY, sentinel=7.0)
        assert call.device_status() == want
        assert (call.out == 7.0).all() and (call.mass == 0).all()
    # a length beyond the block table is clamped and computed
    v = variant(L=16 * b.max_blocks_per_seq + 77)
    call = _run(v, binding.BATCH_PREFILL_ONLY, sentinel=7.0)
    assert call.device_status() == 2 and torch.isfinite(call.mass).all()


def test_single_prompt_reusing_call_and_static_scratch():
    b = W.random_batch(1420, [900], [900], 32, 8, 128, torch.bfloat16, num_probe_heads=4, max_sel_q=3, max_spans=2)
    b.query_sel[0, 0], b.query_sel[0, 1] = 899, 900
    fresh = _run(b, binding.BATCH_PREFILL_ONLY)
    bd = b.to(DEV)
    mass = torch.full_like(fresh.mass, 5.0)
    call = binding.call_from_batch(bd, batch_kind=binding.BATCH_PREFILL_ONLY, plan_mode=binding.PLAN_REUSE, mass=mass,
                                   workspace=fresh.workspace)
    call.launch()
    torch.cuda.synchronize()
    assert torch.equal(bits(call.out), bits(fresh.out))
    assert torch.equal(bits(call.mass[:, :, 0]), bits(fresh.mass[:, :, 0]))
    assert (call.mass[:, :, 1:] == 5.0).all()          # slots without a row: never written by a reusing call
    st = binding.call_from_batch(bd, batch_kind=binding.BATCH_PREFILL_ONLY)
    st.out.fill_(float("nan"))
    st.mass.fill_(float("nan"))
    st.launch_static()
    torch.cuda.synchronize()
    assert torch.equal(bits(st.out), bits(fresh.out)) and torch.equal(bits(st.mass), bits(fresh.mass))


def test_single_prompt_with_new_rows_written_in_the_call():
    b_cpu = W.random_batch(1430, [640], [200], 32, 8, 128, torch.bfloat16, num_probe_heads=4, max_sel_q=2, max_spans=2)
    ref = _run(b_cpu, binding.BATCH_PREFILL_ONLY)
    b = b_cpu.to(DEV)
    k_new = torch.empty(200, 8, 128, dtype=torch.bfloat16, device=DEV)
    v_new = torch.empty_like(k_new)
    for t in range(200):
        pos = 640 - 200 + t
        blk, off = int(b.block_table[0, pos // 16]), pos % 16
        k_new[t], v_new[t] = b.k_cache[blk, :, off], b.v_cache[blk, :, off]
        b.k_cache[blk, :, off] = float("nan")
        b.v_cache[blk, :, off] = float("nan")
    call = binding.call_from_batch(b, batch_kind=binding.BATCH_PREFILL_ONLY, k_new=k_new, v_new=v_new)
    call.launch()
    torch.cuda.synchronize()
    assert torch.equal(bits(call.out), bits(ref.out)) and torch.equal(bits(call.mass), bits(ref.mass))
