"""Offline tuning of the dispatch table for one dense operator whose M is Any, and the
symbolic-versus-static ablation.

The paper tunes a kernel with a symbolic dimension in three steps (Section 3.5): (1) fix the
symbolic dimension at a large enough value (64) and search the configurations, (2) take the
top-k configurations and evaluate them on other shapes (powers of two up to 256), (3) keep the
configuration with the best average, weighted by the workload's shape distribution when it is
known.  Here a "configuration" is a member of the pre-built kernel family: (variant, K split).
`tune_dense` follows those three steps and reports the single best-on-average configuration,
and because this dispatcher can key on the run-time M (the paper's generated dispatch function
keys on the residue only) it also returns the per-M winners as a table for
`nimble_dense_table_set`.

Run on a GPU machine:
    python -m paper_2006_03031_amd.tune --N 3072 --K 768 --epilogue 2 --out table.json
    python -m paper_2006_03031_amd.tune --ablation
"""
from __future__ import annotations

import argparse
import json
from typing import Dict, List, Optional, Sequence, Tuple

import torch

from . import binding as nb
from . import runtime as rt

Config = Tuple[int, int]  # (variant, split_k)


def _time_us(fn, reps: int = 20, rounds: int = 3) -> float:
    """GPU time per call: `reps` launches captured once as a HIP graph (kernel launches only)
    and replayed, so the host's launch cost does not hide differences of a few microseconds."""
    fn()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(reps):
            fn()
    best = float("inf")
    for _ in range(rounds):
        graph.replay()
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        graph.replay()
        e.record()
        torch.cuda.synchronize()
        best = min(best, s.elapsed_time(e) * 1e3 / reps)
    return best


class _Problem:
    def __init__(self, N: int, K: int, epilogue: int, max_m: int):
        self.N, self.K, self.epilogue = N, K, epilogue
        self.x = torch.empty((max_m, K), dtype=torch.bfloat16, device="cuda").uniform_(-1, 1)
        self.w = torch.empty((N, K), dtype=torch.bfloat16, device="cuda").normal_(0, 0.02)
        self.b = torch.empty((N,), dtype=torch.bfloat16, device="cuda").normal_(0, 0.02)
        self.y = torch.empty((max_m, N), dtype=torch.bfloat16, device="cuda")

    def run(self, M: int, force: int = nb.VAR_AUTO) -> None:
        rt.dense(self.x[:M], self.w, self.b, self.epilogue, nb.BF16, force, out=self.y[:M])

    def time(self, M: int, cfg: Optional[Config]) -> float:
        force = nb.VAR_AUTO if cfg is None else (cfg[0] | (cfg[1] << 8) if cfg[1] > 1 else cfg[0])
        try:
            return _time_us(lambda: self.run(M, force))
        except nb.NimbleError:
            return float("inf")  # the configuration cannot run this shape


def candidates(N: int, K: int, M: int) -> List[Config]:
    out: List[Config] = []
    for v in range(1, 7):
        for sk in (1, 2, 4, 8, 16):
            if v < 2 and sk > 1:
                continue
            try:
                nb.dense_plan(M, N, K, nb.EPI_BIAS, nb.BF16, v | (sk << 8) if sk > 1 else v)
            except nb.NimbleError:
                continue
            out.append((v, sk))
    return out


def tune_dense(N: int, K: int, epilogue: int, m_ref: int = 64, m_grid: Sequence[int] = (1, 2, 4, 8, 16, 32, 64, 128, 256),
               top_k: int = 100, weights: Optional[Dict[int, float]] = None, margin: float = 0.03) -> dict:
    """Steps 1-3 of the paper's procedure plus the per-M table.  `weights` maps M to its share of
    the workload (step 3's weighting); `margin` is how much a configuration must beat the
    built-in dispatch before it is written into the table."""
    grid = sorted(set(list(m_grid) + [m_ref]))
    prob = _Problem(N, K, epilogue, max(grid))
    # step 1: every configuration at the reference value of the symbolic dimension
    at_ref = {cfg: prob.time(m_ref, cfg) for cfg in candidates(N, K, m_ref)}
    ranked = sorted((c for c in at_ref if at_ref[c] < float("inf")), key=lambda c: at_ref[c])[:top_k]
    # step 2: the top-k on the other shapes (a configuration that cannot run a shape is out)
    times: Dict[int, Dict[Config, float]] = {}
    for M in grid:
        times[M] = {cfg: prob.time(M, cfg) for cfg in set(ranked) | set(candidates(N, K, M))}
    # step 3: best average (weighted) among the configurations that run every shape
    w = {M: (weights or {}).get(M, 1.0) for M in grid}
    everywhere = [c for c in ranked if all(times[M].get(c, float("inf")) < float("inf") for M in grid)]
    best_avg = min(everywhere, key=lambda c: sum(w[M] * times[M][c] for M in grid)) if everywhere else None
    # per-M winners against the built-in dispatch
    auto = {M: prob.time(M, None) for M in grid}
    table = []
    for i, M in enumerate(grid):
        cfg = min(times[M], key=lambda c: times[M][c])
        if times[M][cfg] < (1.0 - margin) * auto[M]:
            lo = M if i == 0 else (grid[i - 1] + M) // 2 + 1
            hi = M if i == len(grid) - 1 else (M + grid[i + 1]) // 2
            if cfg[0] == 1 and K % 64 != 0:     # the register-layout streaming kernel serves up to 64 rows
                hi = min(hi, 64)
            if lo <= hi:
                table.append([lo, hi, cfg[0], cfg[1]])
    name = lambda c: f"{nb.variant_name(c[0])}/sk{c[1]}"
    return {
        "N": N, "K": K, "epilogue": epilogue, "m_ref": m_ref, "grid": grid,
        "step1_at_m_ref_us": {name(c): round(at_ref[c], 2) for c in ranked},
        "step3_best_average": name(best_avg) if best_avg else None,
        "per_m_us": {str(M): {"auto": round(auto[M], 2), "best": name(min(times[M], key=lambda c: times[M][c])),
                               "best_us": round(min(times[M].values()), 2),
                               "best_average_cfg_us": round(times[M][best_avg], 2) if best_avg else None}
                     for M in grid},
        "table": table,
    }


def load_table(spec: dict) -> None:
    """Install a tuned table (the dict `tune_dense` returns, or its JSON) into the dispatcher."""
    nb.dense_table_set(spec["N"], spec["K"], spec["epilogue"], [tuple(e) for e in spec["table"]])


def ablation(M: int = 128) -> str:
    """Symbolic versus static code generation at M = 128 on the three BERT-base dense layers
    (the experiment of the paper's Figure 3, re-run on this GPU).  Columns:
      static      the r = 0 copy of the 128-row tile: no bounds code, what a kernel compiled
                  for M = 128 would be
      residue     the same tile's r != 0 copy (run at M = 127): the last tile is masked
      big tile    a 256-row tile at M = 128: half of every tile is masked (too few kernels)
      no dispatch the one kernel that handles everything, bounds-checked per element
      dispatch    the dispatch function choosing from the whole family at run time"""
    layers = [("768->2304", 768, 2304, nb.EPI_BIAS), ("768->768", 768, 768, nb.EPI_BIAS),
              ("768->3072 gelu", 768, 3072, nb.EPI_BIAS_GELU_ERF)]
    lines = [f"M = {M}, GPU microseconds per call (20 launches replayed as one HIP graph, best of 3 replays)",
             f"{'layer':<16} {'static':>9} {'residue':>9} {'big tile':>9} {'no dispatch':>12} {'dispatch':>9}  dispatch chose"]
    for name, K, N, epi in layers:
        prob = _Problem(N, K, epi, M)
        t_static = prob.time(M, (4, 1))
        t_res = prob.time(M - 1, (4, 1))
        t_big = prob.time(M, (5, 1))
        t_generic = prob.time(M, (0, 1))
        t_auto = prob.time(M, None)
        p = nb.dense_plan(M, N, K, epi)
        chose = p.name + (f"/sk{p.split_k}" if p.split_k > 1 and p.variant > 1 else "")
        lines.append(f"{name:<16} {t_static:>9.2f} {t_res:>9.2f} {t_big:>9.2f} {t_generic:>12.2f} {t_auto:>9.2f}  {chose}")
    return "\n".join(lines)


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--N", type=int, default=3072)
    ap.add_argument("--K", type=int, default=768)
    ap.add_argument("--epilogue", type=int, default=nb.EPI_BIAS_GELU_ERF)
    ap.add_argument("--m-ref", type=int, default=64)
    ap.add_argument("--grid", type=str, default="1,2,4,8,16,32,64,128,256")
    ap.add_argument("--out", type=str, default="")
    ap.add_argument("--ablation", action="store_true")
    args = ap.parse_args()
    nb.load()
    if args.ablation:
        print(ablation())
        return
    res = tune_dense(args.N, args.K, args.epilogue, args.m_ref, [int(v) for v in args.grid.split(",")])
    text = json.dumps(res, indent=1)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text)
    print(text)


if __name__ == "__main__":
    main()
