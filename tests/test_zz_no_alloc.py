"""hook_attn_probe_static (the entry point that allocates nothing and keeps its work lists in a
static device array) against hook_attn_probe, through the C ABI (needs an MI355X)."""
import ctypes

import pytest
import torch

from paper_2603_06588_amd import binding, workloads as W
from helpers import bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pair(b_cpu, **kw):
    """(out, mass) of the ordinary call and of the static call on the same inputs."""
    b = b_cpu.to(DEV)
    ref = binding.call_from_batch(b, **kw)
    ref.launch()
    torch.cuda.synchronize()
    out = torch.full_like(b.q, float("nan"))
    mass = torch.full_like(ref.mass, float("nan"))
    # a one-byte workspace: the static call must not touch (or need) the caller's
    tiny = torch.zeros(256, dtype=torch.uint8, device=DEV)
    call = binding.call_from_batch(b, out=out, mass=mass, workspace=tiny, **kw)
    call.args.workspace, call.args.workspace_bytes = 0, 0
    call.launch_static()
    torch.cuda.synchronize()
    assert int(tiny.sum()) == 0
    return ref, call


def test_static_scratch_matches_workspace_call_twice_second_smaller():
    # first call: a mixed ragged batch with several decode chunks and prefill items
    big = W.random_batch(210, [2100, 700, 90, 1300, 64, 3000], [1, 700, 1, 1, 64, 2], 8, 2, 128, torch.bfloat16,
                         num_probe_heads=5, max_sel_q=6, max_spans=3)
    ref, got = _pair(big)
    assert torch.equal(bits(got.out), bits(ref.out)) and torch.equal(bits(got.mass), bits(ref.mass))
    # second call, smaller, on the array the first one left behind
    small = W.random_batch(211, [300, 40, 500], [1, 40, 1], 8, 2, 128, torch.bfloat16, num_probe_heads=3,
                           max_sel_q=4, max_spans=2)
    ref, got = _pair(small)
    assert torch.equal(bits(got.out), bits(ref.out)) and torch.equal(bits(got.mass), bits(ref.mass))
    # and against the oracle, to the usual bar
    from helpers import compare_with_oracle
    compare_with_oracle(small, got.out, got.mass, label="static_small")
    # fp32 inputs and the hinted launch sequences take the same route
    f32 = W.random_batch(212, [70, 20], [70, 1], 4, 2, 64, torch.float32, num_probe_heads=2, max_sel_q=3, max_spans=2)
    ref, got = _pair(f32)
    assert torch.equal(bits(got.out), bits(ref.out)) and torch.equal(bits(got.mass), bits(ref.mass))
    dec = W.random_batch(213, [900, 450, 64], [1, 1, 1], 8, 2, 128, torch.bfloat16, num_probe_heads=4, max_sel_q=1,
                         max_spans=2)
    ref, got = _pair(dec, batch_kind=binding.BATCH_DECODE_ONLY)
    assert torch.equal(bits(got.out), bits(ref.out)) and torch.equal(bits(got.mass), bits(ref.mass))


def test_static_scratch_refuses_what_does_not_fit():
    lib = binding.load_library()
    cap = int(lib.hook_attn_probe_static_capacity())
    assert cap == 16 << 20
    # 4096 decode rows with room for 64 k tokens each: the partial records alone exceed the array
    a = binding.HookAttnProbeArgs()
    a.num_seqs, a.total_q, a.num_q_heads, a.num_kv_heads, a.head_dim, a.block_size = 4096, 4096, 32, 8, 128, 16
    a.max_blocks_per_seq, a.num_blocks, a.dtype = 4096, 1 << 20, 0
    for f in ("q", "k_cache", "v_cache", "block_table", "seq_lens", "cu_q_lens", "out"):
        setattr(a, f, 4096)     # never dereferenced: the call is refused on the host
    assert int(lib.hook_attn_probe_workspace_bytes(ctypes.byref(a))) > cap
    assert lib.hook_attn_probe_static(ctypes.byref(a)) == 4
    assert lib.hook_attn_probe_static(None) == 1
