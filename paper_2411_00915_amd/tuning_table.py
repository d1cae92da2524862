"""Shape-keyed table of planner tunables, the counterpart of the hash table shape -> tile
configuration that the paper's offline search fills (section 4.3.2, Algorithm 2).

`autotune.py --out` writes the best setting it measured under the key of the workload's shape;
`apply_for_shape` looks a batch's shape up before `lora_plan` is called and sets the process-wide
tunables accordingly (shapes without an entry keep the built-in defaults).  The key is the batch's
token count rounded up to a power of two, K, N and the largest rank in use: the quantities the
planner's choices depend on.
"""
from __future__ import annotations

import json
import os
from typing import Dict, Optional

from . import binding as B

DEFAULT_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tuning_table.json")


def shape_key(num_tokens: int, k: int, n: int, max_rank: int) -> str:
    bucket = 1
    while bucket < max(int(num_tokens), 1):
        bucket *= 2
    return f"T{bucket}_K{int(k)}_N{int(n)}_R{int(max_rank)}"


def load(path: str = DEFAULT_PATH) -> Dict[str, Dict[str, int]]:
    if not os.path.exists(path):
        return {}
    with open(path) as f:
        table = json.load(f)
    for key, entry in table.items():
        unknown = set(entry) - set(B.TUNING_FIELDS)
        if unknown:
            raise KeyError(f"{path}: entry {key} names unknown tunables {sorted(unknown)}")
    return table


def store(key: str, tunables: Dict[str, int], path: str = DEFAULT_PATH) -> None:
    table = load(path)
    table[key] = {k: int(v) for k, v in sorted(tunables.items())}
    with open(path, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")


def apply_for_shape(num_tokens: int, k: int, n: int, max_rank: int, path: str = DEFAULT_PATH,
                    defaults: Optional[Dict[str, int]] = None) -> Optional[Dict[str, int]]:
    """Set the tunables stored for this shape (on top of `defaults`, if given); returns the entry or None."""
    entry = load(path).get(shape_key(num_tokens, k, n, max_rank))
    if defaults is not None:
        B.lora_tuning_set(**defaults)
    if entry:
        B.lora_tuning_set(**entry)
    return entry
