"""Schedule search (Alg. 1) for the second workload, fused GEMM + LeakyReLU (Sec. 5, Table 3).

The schedule space is the library's table of kernel variants, addressed by their knobs (waves
splitting K, k extent per stage, ring depth, rotated start).  A mutation changes one knob to
another value for which a variant exists (Sec. 3.2's "move one thing by one step", on this
lattice); a candidate is timed only after it has passed the probabilistic test of Sec. 4.2:
its output on random inputs of several shapes must agree with the unmodified (default)
kernel's.  The annealing loop itself is the one shared with the attention search.

  python -m paper_2403_16863_amd.gemm_search [--seed S] [--M 512 --N 512 --K 2048] [--dtype f16]
"""
from __future__ import annotations

import argparse
import json
import random
from typing import Callable, Dict, List, Optional, Sequence, Tuple

from . import inputs as I
from .search import SearchResult, anneal_states

Knobs = Tuple[int, ...]

# shapes of the admission test: the tuned one, and ragged ones in every dimension
TEST_SHAPES = ((512, 512, 2048), (33, 40, 72), (100, 72, 136), (65, 264, 520), (7, 8, 1000), (129, 136, 24))


def neighbours(table: Dict[Knobs, int], x: Knobs) -> List[Knobs]:
    """Variants that differ from x in exactly one knob."""
    return sorted(k for k in table if sum(a != b for a, b in zip(k, x)) == 1)


def propose_from(table: Dict[Knobs, int]) -> Callable[[Knobs, random.Random], Optional[Knobs]]:
    def propose(x: Knobs, rng: random.Random) -> Optional[Knobs]:
        near = neighbours(table, x)
        if not near:                       # an isolated point: any other variant
            near = sorted(k for k in table if k != x)
        return rng.choice(near) if near else None
    return propose


def library_table() -> Dict[Knobs, int]:
    from . import gemm
    return {tuple(gemm.gemm_lrelu_variant_knobs(v)): v for v in range(gemm.gemm_lrelu_num_variants())}


def _device(bits, dtype):
    import numpy as np
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to("cuda")
    return t.view(torch.float16 if dtype == I.F16 else torch.bfloat16)


def admit_against_default(variant: int, dtype: int, samples: int = 12, seed: int = 0, slope: float = I.GEMM_SLOPE) -> bool:
    """Probabilistic test (Sec. 4.2): `samples` random inputs, cycling through TEST_SHAPES and the
    input families; the candidate's output must match the default kernel's to within the
    rounding of the output type (both sum the same products in fp32, in different orders)."""
    import torch
    from . import gemm
    rtol = 2.0 ** -9 if dtype == I.F16 else 2.0 ** -6
    for n in range(samples):
        M, N, K = TEST_SHAPES[n % len(TEST_SHAPES)]
        fam = I.GEMM_FAMILIES[(n // len(TEST_SHAPES)) % len(I.GEMM_FAMILIES)]
        if fam == "large" and dtype == I.F16:
            K = min(K, 1024)
        ab, bb = I.make_gemm(M, N, K, dtype, seed * 1000 + n, fam)
        a, b = _device(ab, dtype), _device(bb, dtype)
        want = torch.full((M, N), float("nan"), dtype=a.dtype, device="cuda")
        got = torch.full((M, N), float("nan"), dtype=a.dtype, device="cuda")
        gemm.gemm_lrelu(a, b, want, slope)
        gemm.gemm_lrelu_variant(a, b, got, slope, variant)
        torch.cuda.synchronize()
        w, g = want.float(), got.float()
        if not bool(torch.isfinite(g).all()):
            return False
        # fp32 summation-order differences: K 2^-24 sum|a||b|, bounded here by the row/column norms
        bound = (a.float().abs().sum(1, keepdim=True) * b.float().abs().amax(0, keepdim=True)) * (2.0 ** -23)
        if not bool(((g - w).abs() <= rtol * w.abs() + bound + 1e-7).all()):
            return False
    return True


def measure_variant(tensors, variant: int, warmup: int = 20, iters: int = 2000, slope: float = I.GEMM_SLOPE) -> float:
    """Microseconds per launch, launches issued back to back."""
    from . import gemm
    a, b, c = tensors
    return gemm.gemm_lrelu_time(a, b, c, slope, variant, warmup, iters) / iters * 1e3


def search(M: int = I.GEMM_M, N: int = I.GEMM_N, K: int = I.GEMM_K, dtype: int = I.F16, seed: int = 0,
           t_max: float = 0.05, t_min: float = 5e-4, cool: float = 1.1, log=None) -> Tuple[SearchResult, Dict[Knobs, int]]:
    import torch
    from . import gemm
    table = library_table()
    by_id = {v: k for k, v in table.items()}
    ab, bb = I.make_gemm(M, N, K, dtype, seed)
    a, b = _device(ab, dtype), _device(bb, dtype)
    c = torch.empty((M, N), dtype=a.dtype, device="cuda")
    x0 = by_id[gemm.gemm_lrelu_default_variant(M, N, K)]
    res = anneal_states(x0, propose_from(table), lambda x: measure_variant((a, b, c), table[x]),
                        lambda x: admit_against_default(table[x], dtype, seed=seed),
                        seed=seed, t_max=t_max, t_min=t_min, cool=cool, log=log)
    return res, table


def main(argv: Optional[Sequence[str]] = None) -> None:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--M", type=int, default=I.GEMM_M)
    ap.add_argument("--N", type=int, default=I.GEMM_N)
    ap.add_argument("--K", type=int, default=I.GEMM_K)
    ap.add_argument("--dtype", choices=("f16", "bf16"), default="f16")
    ap.add_argument("--cool", type=float, default=1.1)
    ap.add_argument("--validate-rounds", type=int, default=7)
    args = ap.parse_args(argv)
    dtype = I.F16 if args.dtype == "f16" else I.BF16

    def log(st):
        t = "-" if st.t_candidate is None else f"{st.t_candidate:.3f}"
        print(f"step {st.step:3d} T={st.temperature:.4f} cand={st.candidate} admitted={st.admitted} "
              f"t={t} accepted={st.accepted}", flush=True)

    res, table = search(args.M, args.N, args.K, dtype, args.seed, cool=args.cool, log=log)
    # the winner against the start, timed again in alternation (a gain has to survive that)
    import torch
    ab, bb = I.make_gemm(args.M, args.N, args.K, dtype, args.seed + 1)
    a, b = _device(ab, dtype), _device(bb, dtype)
    c = torch.empty((args.M, args.N), dtype=a.dtype, device="cuda")
    t_start, t_best = [], []
    for _ in range(args.validate_rounds):
        t_start.append(measure_variant((a, b, c), table[res.x0]))
        t_best.append(measure_variant((a, b, c), table[res.best]))
    t_start.sort()
    t_best.sort()
    med = lambda v: v[len(v) // 2]
    print(json.dumps({"workload": f"gemm_lrelu M{args.M} N{args.N} K{args.K} {args.dtype}", "seed": args.seed,
                      "knobs": ["wk", "bkw", "stages", "rot"], "start": list(res.x0), "t_start_us": res.t0,
                      "best": list(res.best), "t_best_us": res.t_best, "steps": len(res.steps),
                      "measured": len(res.times), "rejected": [list(r) for r in res.rejected],
                      "validated_gain": med(t_start) / med(t_best),
                      "validated_us": {"start": med(t_start), "best": med(t_best)}}))


if __name__ == "__main__":
    main()
