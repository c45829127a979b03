"""Shared comparison helpers for the GPU parity tests (HIP library vs CPU oracle)."""
from __future__ import annotations

from typing import Optional, Sequence

import torch

import oracle

# Tolerances of the parity bar for bf16 inputs: attention output within 2e-2 max-abs of the
# oracle and, because the literal value distribution makes |out| ~ 1e-2, also within 2e-2 of
# max|out_ref|; span masses within 1e-3 absolute.  fp32 inputs are held to 1e-4 / 1e-5.
OUT_ATOL = 2e-2
OUT_RTOL_MAX = 2e-2
MASS_ATOL = 1e-3
F32_OUT_ATOL = 1e-4
F32_MASS_ATOL = 1e-5


def run_hip(b, probe: bool = True):
    from paper_2603_06588_amd import binding
    out, mass = binding.hook_attn_probe_batch(b, probe=probe)
    torch.cuda.synchronize()
    return out, mass


def valid_rows(b) -> torch.Tensor:
    """Global q rows that belong to a sequence with n_i >= 1 (all rows, normally)."""
    cu = b.cu_q_lens.tolist()
    m = torch.zeros(b.total_q, dtype=torch.bool)
    for i in range(b.num_seqs):
        m[cu[i]:cu[i + 1]] = True
    return m


def compare_with_oracle(b_cpu, out_gpu: torch.Tensor, mass_gpu: torch.Tensor,
                        rows: Optional[Sequence[int]] = None, label: str = ""):
    """Element-by-element comparison; returns the error figures."""
    ref_out, ref_mass = oracle.attn_probe_batch(b_cpu, rows=rows)
    got = out_gpu.detach().cpu().double()
    if rows is None:
        sel = valid_rows(b_cpu)
    else:
        sel = torch.zeros(b_cpu.total_q, dtype=torch.bool)
        sel[torch.tensor(list(rows), dtype=torch.long)] = True
    r, g = ref_out[sel], got[sel]
    assert torch.isfinite(g).all(), f"{label}: non-finite attention output"
    err = (r - g).abs().max().item() if r.numel() else 0.0
    ref_max = r.abs().max().item() if r.numel() else 1.0
    f32 = b_cpu.dtype == torch.float32
    atol = F32_OUT_ATOL if f32 else OUT_ATOL
    assert err <= atol, f"{label}: out max-abs error {err:.3e} > {atol}"
    if not f32:
        assert err <= OUT_RTOL_MAX * ref_max, f"{label}: out error {err:.3e} vs max|ref| {ref_max:.3e}"
    merr = 0.0
    if b_cpu.num_probe_heads:
        gm = mass_gpu.detach().cpu().double()
        assert torch.isfinite(gm).all(), f"{label}: non-finite mass"
        merr = (gm - ref_mass).abs().max().item()
        matol = F32_MASS_ATOL if f32 else MASS_ATOL
        assert merr <= matol, f"{label}: mass error {merr:.3e} > {matol}"
    return {"out_err": err, "out_ref_max": ref_max, "mass_err": merr}


def bits(t: torch.Tensor) -> torch.Tensor:
    t = t.detach().cpu().contiguous()
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)
