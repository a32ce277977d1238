"""Deployment of searched schedules (paper Sec. 4.1).

The searches run offline and leave two kinds of results: a validated ranking of the schedule
variants per workload (`search_store/ranking_<workload>.json`, written by
`search.py --store-ranking`) and, from the instruction-level search, a code object with a small
description next to it (`sip.py --keep-codeobj FILE` writes FILE and FILE.json).  This module
turns either into an entry of the library's deployment table, after which `attn_fwd` launches
the searched schedule for the shapes it was searched on: chosen once, no cost per call.

A ranking is deployed only if its best variant differs from the library default and its
validated gain exceeds `min_gain` (the timing noise of the boxes is 1 to 2 %; a "gain" below
that is not one).  Host logic around the C-ABI calls; nothing here touches the device.
"""
import glob
import json
import os
import re
import shutil
from typing import List, Optional

from . import binding as B
from . import inputs as I

STORE_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "search_store")

_LABEL = re.compile(r"B(\d+) H(\d+) N(\d+) d(\d+) (causal|full) (f16|bf16)")


def shape_of_ranking(summary: dict) -> dict:
    """{"N", "d", "causal", "dtype"} of a stored ranking (its "shape" entry, or parsed from the
    workload label of files written before that entry existed)."""
    if "shape" in summary:
        return summary["shape"]
    m = _LABEL.search(summary["workload"])
    if not m:
        raise ValueError(f"cannot read the shape from {summary['workload']!r}")
    return {"B": int(m.group(1)), "H": int(m.group(2)), "N": int(m.group(3)), "d": int(m.group(4)),
            "causal": m.group(5) == "causal", "dtype": I.F16 if m.group(6) == "f16" else I.BF16}


def default_range(N: int):
    """Sequence lengths a result measured at N is applied to: from N/2 (exclusive) to 2N
    (exclusive), the neighbourhood in which the same loop dominates the run time."""
    return N // 2 + 1, 2 * N - 1


def deploy_ranking(path: str, n_min: Optional[int] = None, n_max: Optional[int] = None,
                   min_gain: float = 1.02) -> Optional[dict]:
    """Deploys the best variant of one stored ranking; returns what was deployed, or None when
    the ranking's best is the library default or its gain is inside the noise."""
    with open(path) as fh:
        summary = json.load(fh)
    shape = shape_of_ranking(summary)
    best, gain = int(summary["best_variant"]), float(summary["best_vs_default"])
    default = B.attn_default_variant(shape["N"], shape["d"], shape["dtype"], shape["causal"])
    if best == default or gain < min_gain:
        return None
    lo, hi = default_range(shape["N"])
    lo, hi = (lo if n_min is None else n_min), (hi if n_max is None else n_max)
    B.attn_deploy_variant(best, shape["d"], shape["dtype"], shape["causal"], lo, hi)
    return {"ranking": os.path.basename(path), "variant": best, "gain": gain, "d": shape["d"], "dtype": shape["dtype"],
            "causal": shape["causal"], "n_min": lo, "n_max": hi}


def deploy_stored_rankings(store_dir: str = STORE_DIR, min_gain: float = 1.02) -> List[dict]:
    """Deploys every stored ranking that has something to deploy (sorted by file name, so a
    later file wins where ranges overlap)."""
    done = []
    for path in sorted(glob.glob(os.path.join(store_dir, "ranking_*.json"))):
        r = deploy_ranking(path, min_gain=min_gain)
        if r:
            done.append(r)
    return done


def save_codeobj(co_path: str, dest: str, kernel_name: str, variant: int, workload, validated_gain: Optional[float]) -> None:
    """Keeps a searched code object: copies it to `dest` and writes `dest`.json with what
    `deploy_codeobj_file` needs to load it."""
    shutil.copyfile(co_path, dest)
    with open(dest + ".json", "w") as fh:
        json.dump({"kernel_name": kernel_name, "variant": int(variant), "N": workload.N, "d": workload.d,
                   "dtype": int(workload.dtype), "causal": bool(workload.causal), "workload": workload.label,
                   "validated_gain": validated_gain}, fh, indent=1)
        fh.write("\n")


def deploy_codeobj_file(co_path: str, n_min: Optional[int] = None, n_max: Optional[int] = None) -> int:
    """Loads a kept code object and makes it what attn_fwd launches for its shape class;
    returns the handle (keep it loaded for as long as it is deployed)."""
    with open(co_path + ".json") as fh:
        meta = json.load(fh)
    h = B.attn_codeobj_load(co_path, meta["kernel_name"], meta["variant"], meta["d"], meta["dtype"], meta["causal"])
    lo, hi = default_range(meta["N"])
    try:
        B.attn_deploy_codeobj(h, lo if n_min is None else n_min, hi if n_max is None else n_max)
    except B.AttnError:
        B.attn_codeobj_unload(h)
        raise
    return h
