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
