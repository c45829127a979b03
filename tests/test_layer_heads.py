"""The layer/heads string parser: reference parser pinned by the paper's printed example, the
library's C parser checked against the reference (no GPU needed)."""
import ctypes
import json
import os
import random

import pytest

from oracle.config import parse_layer_heads as ref_parse

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2603_06588_amd import binding as b, build
    if build.lib_is_stale():
        build.build_lib()
    return b


def _golden():
    lines = [l for l in open(os.path.join(ROOT, "tests", "golden", "layer_heads_example.txt")).read().splitlines()
             if l and not l.startswith("#")]
    return lines[0], {int(k): v for k, v in json.loads(lines[1]).items()}


def test_reference_parser_matches_the_papers_example():
    text, want = _golden()
    assert ref_parse(text) == want
    assert ref_parse("") == {}
    assert ref_parse(" 3 : 1 , 2 ;; 3:7 ") == {3: [1, 2, 7]}
    for bad in ["3", "3:", "a:1", "3:1:2", "-1:2"]:
        with pytest.raises(ValueError):
            ref_parse(bad)


def _as_dict(pairs):
    out = {}
    for l, h in pairs:
        out.setdefault(l, []).append(h)
    return out


def test_library_parser_matches_reference(binding):
    text, want = _golden()
    assert _as_dict(binding.parse_layer_heads(text)) == want
    rng = random.Random(0)
    for _ in range(200):
        parts = []
        for _ in range(rng.randint(0, 6)):
            layer = rng.randint(0, 80)
            heads = [rng.randint(0, 127) for _ in range(rng.randint(1, 7))]
            sep = rng.choice([",", " ,", ", "])
            parts.append(f"{layer}{rng.choice([':', ' : '])}{sep.join(map(str, heads))}")
        s = rng.choice([";", " ; ", ";;"]).join(parts)
        assert _as_dict(binding.parse_layer_heads(s)) == ref_parse(s)
    for bad in ["3", "3:", "a:1", "3:1:2", "-1:2", "3:1,", "3:1;x", "99999999999:1"]:
        with pytest.raises(binding.HookError):
            binding.parse_layer_heads(bad)
    # capacity handling: count is reported, nothing past capacity is written
    lib = binding.load_library()
    cnt = ctypes.c_int32(0)
    l2, h2 = (ctypes.c_int32 * 2)(), (ctypes.c_int32 * 2)()
    assert lib.hook_parse_layer_heads(text.encode(), l2, h2, 2, ctypes.byref(cnt)) == 4
    assert cnt.value == 4 and list(l2) == [0, 0] and list(h2) == [0, 3]


def test_probe_heads_for_layer(binding):
    pairs = binding.parse_layer_heads("8:14,1,13,15;7:20;8:1")
    assert binding.probe_heads_for_layer(pairs, 8).tolist() == [1, 13, 14, 15]
    assert binding.probe_heads_for_layer(pairs, 7).tolist() == [20]
    assert binding.probe_heads_for_layer(pairs, 9).numel() == 0
