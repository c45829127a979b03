"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared
symbol, and rejects malformed arguments before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2603_06588_amd import binding as b, build
    if build.lib_is_stale():
        build.build_lib()
    return b


def _header_struct_fields(struct_name: str):
    """Field names of a struct declared in include/hook_api.h, in declaration order."""
    header = open(os.path.join(ROOT, "include", "hook_api.h")).read()
    body = header[header.index(f"typedef struct {struct_name} {{"):header.index(f"}} {struct_name};")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for stmt in body.split("{", 1)[1].split(";"):
        stmt = stmt.strip()
        if not stmt:
            continue
        decl = stmt.split(None, 1)[1] if not stmt.startswith("const") else stmt.split(None, 2)[2]
        names += [n.strip().lstrip("*").strip() for n in decl.split(",")]
    return names


def test_exports_every_declared_symbol(binding):
    header = open(os.path.join(ROOT, "include", "hook_api.h")).read()
    declared = set(re.findall(r"\b(hook_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    lib = binding.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert binding.version() >= 1
    assert binding.status_string(0) == "ok"


def test_measurement_library_exports_its_header_and_the_product_does_not(binding):
    from paper_2603_06588_amd import benchlib
    header = open(os.path.join(ROOT, "include", "hook_bench.h")).read()
    declared = set(re.findall(r"\b(hook_bench_[a-z0-9_]+)\s*\(", header))
    assert declared == set(benchlib.EXPORTS)
    lib = benchlib.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    product = binding.load_library()
    for name in declared:
        assert not hasattr(product, name), name     # measurement aids stay out of the product ABI
    # the dynamic symbol table of the product holds the declared calls and nothing else of ours
    import subprocess
    syms = subprocess.run(["nm", "-D", "--defined-only", binding.LIB_PATH], capture_output=True, text=True).stdout
    ours = {ln.split()[-1] for ln in syms.splitlines() if " T " in ln}
    assert ours == set(binding.EXPORTS), ours ^ set(binding.EXPORTS)


def test_args_struct_matches_header_field_order(binding):
    assert _header_struct_fields("hook_attn_probe_args") == [f[0] for f in binding.HookAttnProbeArgs._fields_]


def test_capture_struct_matches_header_field_order(binding):
    names = _header_struct_fields("hook_capture_qk_args")
    assert names == [f[0] for f in binding.HookCaptureQkArgs._fields_]
    lib = binding.load_library()
    a = binding.HookCaptureQkArgs()
    assert lib.hook_capture_qk(None) == 1
    a.num_seqs, a.num_q_heads, a.num_kv_heads, a.head_dim, a.block_size = 1, 8, 2, 128, 32
    a.max_blocks_per_seq, a.num_blocks = 4, 4
    assert lib.hook_capture_qk(ctypes.byref(a)) == 3          # block size
    a.block_size = 16
    a.num_probe_heads, a.max_sel_q = 2, 1
    assert lib.hook_capture_qk(ctypes.byref(a)) == 1          # null arrays


def test_kv_write_struct_and_argument_checks(binding):
    names = _header_struct_fields("hook_kv_write_args")
    assert names == [f[0] for f in binding.HookKvWriteArgs._fields_]
    lib = binding.load_library()
    assert lib.hook_kv_write(None) == 1
    a = binding.HookKvWriteArgs()
    a.num_seqs, a.total_q, a.num_kv_heads, a.head_dim, a.block_size = 1, 4, 2, 128, 16
    a.max_blocks_per_seq, a.num_blocks = 4, 4
    assert lib.hook_kv_write(ctypes.byref(a)) == 1             # null arrays
    a.block_size = 8
    assert lib.hook_kv_write(ctypes.byref(a)) == 3             # block size
    a.block_size, a.total_q = 16, 0
    assert lib.hook_kv_write(ctypes.byref(a)) == 0             # nothing to write


def test_span_mass_argument_checks(binding):
    lib = binding.load_library()
    assert lib.hook_span_mass(None) == 1
    a = binding.HookAttnProbeArgs()
    a.num_seqs, a.total_q, a.num_q_heads, a.num_kv_heads, a.head_dim = 1, 4, 8, 2, 128
    a.block_size, a.max_blocks_per_seq, a.num_blocks, a.dtype = 16, 4, 4, 0
    a.num_probe_heads, a.max_sel_q, a.max_spans = 2, 4, 1025
    assert lib.hook_span_mass(ctypes.byref(a)) == 3            # more spans than HOOK_MAX_SPANS_WIDE
    a.max_spans = 100
    assert lib.hook_span_mass(ctypes.byref(a)) == 1            # null arrays
    a.dtype = 1
    assert lib.hook_span_mass(ctypes.byref(a)) == 3            # fp32 inputs are not supported here
    a.dtype, a.num_probe_heads = 0, 0
    assert lib.hook_span_mass(ctypes.byref(a)) == 2            # nothing to probe
    # scratch size of the split form: none for a null struct, grows with rows and context length
    assert lib.hook_span_mass_workspace_bytes(None) == 0
    a.num_probe_heads, a.max_blocks_per_seq = 2, 64
    small = lib.hook_span_mass_workspace_bytes(ctypes.byref(a))
    a.max_blocks_per_seq, a.max_sel_q = 1024, 64
    big = lib.hook_span_mass_workspace_bytes(ctypes.byref(a))
    assert big > small > 0 and small % 8 == 0 and big % 8 == 0


def test_reduce_struct_and_argument_checks(binding):
    names = _header_struct_fields("hook_reduce_args")
    assert names == [f[0] for f in binding.HookReduceArgs._fields_]
    lib = binding.load_library()
    assert lib.hook_reduce_mass(None) == 1
    a = binding.HookReduceArgs()
    a.num_seqs, a.num_probe_heads, a.max_sel_q, a.max_spans = 2, 4, 1, 2
    a.mode, a.span_a, a.span_b = 1, 0, 1
    assert lib.hook_reduce_mass(ctypes.byref(a)) == 1          # null mass / scores
    a.span_b = 2
    assert lib.hook_reduce_mass(ctypes.byref(a)) == 2          # span index out of range
    a.span_b, a.mode = 1, 7
    assert lib.hook_reduce_mass(ctypes.byref(a)) == 3          # unknown mode
    a.mode, a.max_spans = 0, 1025
    assert lib.hook_reduce_mass(ctypes.byref(a)) == 2          # more spans than the compiled bound
    a.max_spans, a.num_seqs = 2, 0
    assert lib.hook_reduce_mass(ctypes.byref(a)) == 0          # empty batch: nothing to do


def _args(binding, **kw):
    a = binding.HookAttnProbeArgs()
    base = dict(num_seqs=2, total_q=10, num_q_heads=8, num_kv_heads=2, head_dim=128, block_size=16,
                max_blocks_per_seq=4, num_blocks=16, dtype=0, scale=0.0)
    base.update(kw)
    for k, v in base.items():
        setattr(a, k, v)
    return a


def test_rejects_bad_arguments_before_launch(binding):
    lib = binding.load_library()
    call = lambda a: lib.hook_attn_probe(ctypes.byref(a))
    assert lib.hook_attn_probe(None) == 1
    assert call(_args(binding, num_q_heads=6, num_kv_heads=4)) == 2       # Hq % Hkv != 0
    assert call(_args(binding, head_dim=96)) == 3
    assert call(_args(binding, block_size=32)) == 3
    assert call(_args(binding, dtype=7)) == 3
    assert call(_args(binding, num_seqs=-1)) == 2
    assert call(_args(binding, plan_mode=2)) == 2
    assert call(_args(binding)) == 1                                      # null tensors
    a = _args(binding, num_probe_heads=2, max_sel_q=1, max_spans=9)
    assert call(a) == 3                                                   # too many spans
    a = _args(binding, num_probe_heads=2, max_sel_q=1, max_spans=1)
    assert call(a) == 1                                                   # probe arrays null
    a = _args(binding, num_probe_heads=9)
    assert call(a) == 2                                                   # more probe heads than heads
    # everything non-null but no workspace
    a = _args(binding)
    for f in ("q", "k_cache", "v_cache", "block_table", "seq_lens", "cu_q_lens", "out"):
        setattr(a, f, 4096)
    assert call(a) == 4
    a.workspace, a.workspace_bytes = 4096 + 8, 1 << 30                    # misaligned
    assert call(a) == 4
    assert lib.hook_attn_probe_workspace_bytes(ctypes.byref(_args(binding, head_dim=96))) == 0
    assert lib.hook_attn_probe_workspace_bytes(ctypes.byref(_args(binding))) > 0
    # capacities whose launch grid would not fit 31 bits are refused, not truncated
    a = _args(binding, num_seqs=1 << 20, total_q=1 << 20, max_blocks_per_seq=1 << 20, num_blocks=1 << 20)
    for f in ("q", "k_cache", "v_cache", "block_table", "seq_lens", "cu_q_lens", "out"):
        setattr(a, f, 4096)
    a.workspace, a.workspace_bytes = 4096, 1 << 62
    assert call(a) == 3
    # empty batch is a no-op
    assert call(_args(binding, num_seqs=0, total_q=0)) == 0


def test_validate_argument_checks(binding):
    lib = binding.load_library()
    bits = ctypes.c_int32(7)
    assert lib.hook_attn_probe_validate(None, ctypes.byref(bits)) == 1
    a = _args(binding)
    assert lib.hook_attn_probe_validate(ctypes.byref(a), None) == 1
    assert lib.hook_attn_probe_validate(ctypes.byref(a), ctypes.byref(bits)) == 1      # null arrays
    assert bits.value == 0
    for f in ("block_table", "seq_lens", "cu_q_lens"):
        setattr(a, f, 4096)
    assert lib.hook_attn_probe_validate(ctypes.byref(a), ctypes.byref(bits)) == 4      # no workspace
    a.batch_kind = 5
    assert lib.hook_attn_probe_validate(ctypes.byref(a), ctypes.byref(bits)) == 2


def test_steer_argument_checks(binding):
    lib = binding.load_library()
    assert lib.hook_steer(None, None, 1.0, None, 4, 64, 0, None) == 1
    assert lib.hook_steer(4096, 4096, 1.0, 4096, 4, 60, 0, None) == 3     # not a multiple of 8
    assert lib.hook_steer(4096, 4096, 1.0, 4096, 4, 64, 5, None) == 3
    assert lib.hook_steer(4096, 4096, 1.0, 4096, -1, 64, 0, None) == 2
    assert lib.hook_steer(4096, 4096, 0.0, 4096, 4, 64, 0, None) == 0     # alpha = 0: nothing launched
    assert lib.hook_steer(None, None, 1.0, None, 0, 64, 0, None) == 0


def test_workspace_size_grows_with_decode_capacity(binding):
    lib = binding.load_library()
    small = lib.hook_attn_probe_workspace_bytes(ctypes.byref(_args(binding, num_seqs=4, total_q=4, max_blocks_per_seq=64)))
    big = lib.hook_attn_probe_workspace_bytes(ctypes.byref(_args(binding, num_seqs=4, total_q=4, max_blocks_per_seq=512)))
    assert big > small > 0


def test_plain_c_program_compiles_links_and_runs(binding, tmp_path):
    """include/hook_api.h is a C header: a C99 program (tests/c_abi_client.c) built with gcc -pedantic
    links every entry point and gets the documented answers from the host-side checks."""
    import subprocess
    binding.load_library()
    libdir = os.path.dirname(binding.LIB_PATH)
    exe = str(tmp_path / "c_abi_client")
    cc = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror",
                         "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c_abi_client.c"),
                         "-o", exe, "-L", libdir, "-lhook", f"-Wl,-rpath,{libdir}"],
                        capture_output=True, text=True)
    assert cc.returncode == 0, cc.stdout + cc.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert run.returncode == 0, run.stdout + run.stderr
