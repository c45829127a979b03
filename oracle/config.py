"""Reference parser for the layer/heads string of the paper's worker (TEST INFRASTRUCTURE ONLY).

Section 2.1 (worker listing, `_parse_layer_heads`): the environment string
`'<layer>:<head>,<head>,...;<layer>:...'` maps to `{layer: [heads...]}`; the paper prints one
worked example, kept in tests/golden/layer_heads_example.txt.  Plain Python, no shared code
with the library's C parser.
"""
from typing import Dict, List


def parse_layer_heads(text: str) -> Dict[int, List[int]]:
    out: Dict[int, List[int]] = {}
    text = text.strip()
    if not text:
        return out
    for part in text.split(";"):
        part = part.strip()
        if not part:
            continue
        if part.count(":") != 1:
            raise ValueError(f"expected '<layer>:<heads>' in {part!r}")
        layer_s, heads_s = part.split(":")
        layer = int(layer_s)
        heads = [int(h) for h in heads_s.split(",") if h.strip() != ""]
        if layer < 0 or any(h < 0 for h in heads) or not heads:
            raise ValueError(f"bad entry {part!r}")
        out.setdefault(layer, []).extend(heads)
    return out


def parse_config_json(text: str):
    """Section 2 (config file example): ([(layer, head), ...] in file order, hookq_mode or None),
    read with the standard json module."""
    import json
    doc = json.loads(text)
    if not isinstance(doc, dict):
        raise ValueError("top level must be an object")
    pairs = []
    params = doc.get("params")
    if isinstance(params, dict) and "important_heads" in params:
        for item in params["important_heads"]:
            if (not isinstance(item, list) or len(item) != 2 or
                    any(isinstance(x, bool) or not isinstance(x, int) or x < 0 for x in item)):
                raise ValueError(f"bad pair {item!r}")
            pairs.append((item[0], item[1]))
    mode = None
    hookq = doc.get("hookq")
    if isinstance(hookq, dict) and "hookq_mode" in hookq:
        mode = hookq["hookq_mode"]
        if mode not in ("last_token", "all_tokens"):
            raise ValueError(f"unknown hookq_mode {mode!r}")
    return pairs, mode
