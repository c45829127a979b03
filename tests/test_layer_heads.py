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


# ---- JSON configuration file ----

def _config_golden():
    text = open(os.path.join(ROOT, "tests", "golden", "config_example.json")).read()
    lines = [l for l in open(os.path.join(ROOT, "tests", "golden", "config_example_expected.txt")).read().splitlines()
             if l and not l.startswith("#")]
    return text, ref_parse(lines[0]), lines[1], int(lines[2])


def test_reference_config_reader_matches_the_papers_example():
    from oracle.config import parse_config_json
    text, want_map, want_mode, want_n = _config_golden()
    pairs, mode = parse_config_json(text)
    assert len(pairs) == want_n and mode == want_mode
    assert _as_dict(pairs) == want_map
    assert pairs[0] == (6, 9) and pairs[-1] == (19, 1)
    assert parse_config_json('{"params": {}, "x": [1, {"hookq_mode": "all_tokens"}]}') == ([], None)
    assert parse_config_json('{"hookq": {"hookq_mode": "all_tokens"}}') == ([], "all_tokens")
    for bad in ['[1]', '{"params": {"important_heads": [[1]]}}', '{"params": {"important_heads": [[1, -2]]}}',
                '{"params": {"important_heads": [[1, 2.5]]}}', '{"hookq": {"hookq_mode": "first"}}']:
        with pytest.raises(ValueError):
            parse_config_json(bad)


def test_library_config_reader_matches_reference(binding):
    from oracle.config import parse_config_json
    text, want_map, want_mode, want_n = _config_golden()
    pairs, mode = binding.parse_config_json(text)
    assert (pairs, mode) == parse_config_json(text)
    assert len(pairs) == want_n and _as_dict(pairs) == want_map and mode == want_mode
    rng = random.Random(1)

    def junk(depth=0):
        k = rng.randint(0, 6 if depth < 3 else 4)
        if k == 0:
            return rng.randint(-50, 50)
        if k == 1:
            return rng.choice([True, False, None, 1.5e-3, -2.25, 'a "quoted" str', "important_heads", ""])
        if k == 2:
            return rng.random() * 1e6
        if k == 3:
            return "x" * rng.randint(0, 5)
        if k == 4:
            return [rng.randint(0, 9) for _ in range(rng.randint(0, 4))]
        if k == 5:
            return [junk(depth + 1) for _ in range(rng.randint(0, 3))]
        return {f"k{j}": junk(depth + 1) for j in range(rng.randint(0, 3))}

    for _ in range(200):
        doc = {f"top{j}": junk() for j in range(rng.randint(0, 3))}
        if rng.random() < 0.8:
            doc["params"] = {"other": junk(), "important_heads": [[rng.randint(0, 80), rng.randint(0, 127)]
                                                                  for _ in range(rng.randint(0, 30))]}
        if rng.random() < 0.7:
            doc["hookq"] = {"hookq_mode": rng.choice(["last_token", "all_tokens"]), "more": junk()}
        if rng.random() < 0.3:
            doc["decoy"] = {"params": {"important_heads": [[1, 2]]}, "hookq": {"hookq_mode": "all_tokens"}}
        items = list(doc.items())
        rng.shuffle(items)
        s = json.dumps(dict(items), indent=rng.choice([None, 0, 2]))
        assert binding.parse_config_json(s) == parse_config_json(s), s
    for bad in ['', '[1]', '{"a": }', '{"a": 1,}', '{"params": {"important_heads": [[1]]}}', '{"a": 1} x',
                '{"params": {"important_heads": [[1, -2]]}}', '{"params": {"important_heads": [[1, 2.5]]}}',
                '{"params": {"important_heads": [[1, 2], ]}}', '{"hookq": {"hookq_mode": "first"}}', '{"a": tru}']:
        with pytest.raises(binding.HookError):
            binding.parse_config_json(bad)
