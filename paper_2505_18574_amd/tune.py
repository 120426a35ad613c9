"""Search over the launch plans (kernel / block tile, K split) of the GEMM and convolution entry points.

This is the part of the paper's optimisation loop that needs no language model: candidates are run on the
device, kept only if their output is still correct, and ranked by measured latency; the best few seed the
next iteration (beam search, Section 3.3).  A plan found for one shape can seed the search for a related
shape, which then looks only at that plan and its neighbours (schedule reuse, Sections 3.5 and 5).

A candidate here is a (tile, splits) pair of ac_gemm_i8_planned / ac_gemm_bf16_planned / ac_conv2d_i8_planned.  Every candidate is
run through the C ABI; nothing is computed on the host.  The correctness gate is a callable supplied by the
caller (the tests pass one that compares against the CPU oracle); without one, a candidate must reproduce the
library's own unplanned result -- bit for bit for int8, to a relative Frobenius error of 1e-5 for bf16 (two
fp32 summation orders of the same products).
"""
from __future__ import annotations

import dataclasses
import json
from typing import Callable, Dict, Iterable, List, Optional, Sequence, Tuple

import torch

from . import ops

Plan = Tuple[int, int]  # (tile code, splits)
TILES = (64, 128, 192, 256)  # tile codes in order of area; 192 is the 256 x 128 (rows x columns) tile
TILE_DIMS = {32: (32, 32), 64: (64, 64), 128: (128, 128), 192: (256, 128), 256: (256, 256), 160: (128, 64), 320: (256, 64)}
# int8 only: one wave per 32 x 32 tile, for launches of a few microseconds; K in whole 64-byte tiles
SMALL_TILES = (32,)
# int8 only: the weight-stationary kernel (128- / 256-row tiles, 64 columns, all of K resident in LDS, no K split)
WS_TILES = (160, 320)
WS_MAX_K = {160: 2048, 320: 1536}
# convolutions only (kind "conv"): the patch kernel with 128- / 256-pixel work units; the library refuses it for
# geometries it does not fit, and a refused plan simply drops out of the search
HALO_TILES = (161, 321)
MAX_WORKGROUPS = 8192          # more slices than this only add reduction traffic
MAX_WORKSPACE_BYTES = 1 << 30  # partial sums (int32 / fp32, splits * M * N * 4 bytes) the tuner is willing to allocate


def k_tiles(kind: str, K: int, tile: int) -> int:
    """K tiles of the kernel behind `tile`: 64 bytes of K per tile for the 256 tile, 128 bytes otherwise."""
    kbytes = K * (2 if kind == "bf16" else 1)
    ktb = 64 if tile in (256, 32) else 128
    return (kbytes + ktb - 1) // ktb


def normalise(kind: str, K: int, plan: Plan) -> Plan:
    """The plan the library actually runs: slices hold whole K tiles, so several split counts coincide."""
    tile, splits = plan
    nkt = k_tiles(kind, K, tile)
    if splits <= 1 or nkt <= 1:
        return tile, 1
    per = (nkt + splits - 1) // splits
    return tile, max(1, (nkt + per - 1) // per)


def valid(kind: str, M: int, N: int, K: int, plan: Plan) -> bool:
    tile, splits = plan
    if tile in SMALL_TILES and not (kind in ("i8", "conv") and K >= 64 and K % 64 == 0):
        return False
    if tile in WS_TILES:
        return kind in ("i8", "conv") and splits == 1 and 1 <= K <= WS_MAX_K[tile]
    if tile in HALO_TILES:
        return kind == "conv" and splits == 1
    if tile not in TILES + SMALL_TILES or splits < 1 or (splits > 1 and splits > k_tiles(kind, K, tile)):
        return False
    bm, bn = TILE_DIMS[tile]
    workgroups = ((M + bm - 1) // bm) * ((N + bn - 1) // bn) * splits
    if splits > 1 and workgroups > MAX_WORKGROUPS:
        return False
    if splits > 1 and splits * M * N * 4 > MAX_WORKSPACE_BYTES:
        return False
    return True


def all_plans(kind: str, M: int, N: int, K: int) -> List[Plan]:
    """Every tile with every power-of-two split that is valid for the shape."""
    out: List[Plan] = []
    for tile in SMALL_TILES + TILES:
        s = 1
        while valid(kind, M, N, K, (tile, s)):
            q = normalise(kind, K, (tile, s))
            if q not in out:
                out.append(q)
            s *= 2
    out += [(t, 1) for t in WS_TILES + HALO_TILES if valid(kind, M, N, K, (t, 1))]
    return out


def seed_plans(kind: str, M: int, N: int, K: int, auto: Plan, workgroups: int = 256) -> List[Plan]:
    """Starting points of the beam: the library's own plan, plus for every tile the smallest power-of-two split
    that gives every compute unit a workgroup (the beam only ever moves to a faster neighbour, so it needs a
    start on each side of the tile-size trade-off)."""
    out = [normalise(kind, K, auto)]
    for tile in TILES:
        bm, bn = TILE_DIMS[tile]
        tiles = ((M + bm - 1) // bm) * ((N + bn - 1) // bn)
        s = 1
        while tiles * s < workgroups and valid(kind, M, N, K, (tile, s * 2)):
            s *= 2
        q = normalise(kind, K, (tile, s))
        if valid(kind, M, N, K, q) and q not in out:
            out.append(q)
    out += [(t, 1) for t in WS_TILES + HALO_TILES if valid(kind, M, N, K, (t, 1)) and (t, 1) not in out]
    return out


def neighbours(kind: str, M: int, N: int, K: int, plan: Plan) -> List[Plan]:
    """One step from `plan`: the next tile code up or down, half or twice the split."""
    tile, splits = plan
    if tile in SMALL_TILES:  # its neighbours: the smallest tile of the tiled kernels at the same split, half or twice the split
        cand = [(64, splits), (tile, max(1, splits // 2)), (tile, splits * 2)]
    elif tile in WS_TILES:  # its neighbours: the other row-tile height, and the tiled kernels of similar height
        cand = [(WS_TILES[1 - WS_TILES.index(tile)], 1), (64, 1), (192, 1)] + [(t, 1) for t in HALO_TILES]
    elif tile in HALO_TILES:  # the other unit size, the other resident-operand kernel, the tiled kernels
        cand = [(HALO_TILES[1 - HALO_TILES.index(tile)], 1)] + [(t, 1) for t in WS_TILES] + [(64, 1), (192, 1)]
    else:
        i = TILES.index(tile)
        cand = [(TILES[j], splits) for j in (i - 1, i + 1) if 0 <= j < len(TILES)]
        cand += [(tile, max(1, splits // 2)), (tile, splits * 2)]
        if tile == 64:
            cand += [(t, splits) for t in SMALL_TILES]
    out: List[Plan] = []
    for c in cand:
        if valid(kind, M, N, K, c):
            c = normalise(kind, K, c)
            if c != plan and c not in out:
                out.append(c)
    return out


def measure_us(fn: Callable[[], None], min_ms: float = 2.0, warmup: int = 3, reps: int = 20) -> float:
    """Microseconds per call of `fn`, which enqueues device work on the current stream.

    `reps` calls are captured into one HIP graph and the graph is replayed between two device events until
    the timed region is at least `min_ms` long: a graph launch keeps the host's per-call cost (tens of
    microseconds from Python) out of the figure, which matters for kernels that run only a few microseconds."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for _ in range(warmup):
            fn()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(reps):
                fn()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        replays = 1
        while True:
            graph.replay()  # settle clocks and caches before the timed replays
            start.record()
            for _ in range(replays):
                graph.replay()
            stop.record()
            stop.synchronize()
            ms = start.elapsed_time(stop)
            if ms >= min_ms or replays >= 1024:
                break
            replays *= 4
    torch.cuda.current_stream().wait_stream(side)
    return ms * 1e3 / (reps * replays)


@dataclasses.dataclass
class Trial:
    plan: Plan
    correct: bool
    us: Optional[float]  # None when the candidate failed the correctness gate


@dataclasses.dataclass
class TuneResult:
    best: Plan
    best_us: float
    trials: List[Trial]


class _Problem:
    """One GEMM call with its operands bound; run(plan) launches it, reference() launches the unplanned call."""

    def __init__(self, kind: str, M: int, N: int, K: int, run, reference, out, exact: bool,
                 sync=torch.cuda.synchronize, measure=measure_us, confirm=None):
        self.kind, self.M, self.N, self.K = kind, M, N, K
        self.run, self.reference, self.out, self.exact = run, reference, out, exact
        self.sync, self.measure = sync, measure  # replaceable so that the search logic can be tested without a device
        # the longer measurement that decides between the finalists of a search: a 2 ms region ranks a whole
        # candidate set quickly, but it catches the clocks of a large kernel still settling
        self.confirm = confirm or (measure if measure is not measure_us else (lambda fn: measure_us(fn, min_ms=20.0)))


def _default_gate(prob: _Problem) -> Callable[[torch.Tensor], bool]:
    prob.reference()
    prob.sync()
    want = prob.out.clone()
    if prob.exact:
        return lambda got: bool(torch.equal(got, want))
    den = want.double().norm()
    return lambda got: bool((got.double() - want.double()).norm() <= 1e-5 * den)


def _evaluate(prob: _Problem, plan: Plan, gate, seen: Dict[Plan, Trial]) -> Trial:
    if plan in seen:
        return seen[plan]
    prob.out.zero_()
    try:
        prob.run(plan)
    except ops.AcError:  # a plan these operands cannot take (alignment, bias layout): not a candidate
        seen[plan] = Trial(plan, False, None)
        return seen[plan]
    prob.sync()
    ok = bool(gate(prob.out))
    trial = Trial(plan, ok, prob.measure(lambda: prob.run(plan)) if ok else None)
    seen[plan] = trial
    return trial


FINALISTS = 3  # candidates of a search that are measured again, longer, before the best is named


def _search(prob: _Problem, gate, start: Sequence[Plan], beam: int, iterations: int, exhaustive: bool) -> TuneResult:
    gate = gate or _default_gate(prob)
    seen: Dict[Plan, Trial] = {}
    kind, M, N, K = prob.kind, prob.M, prob.N, prob.K
    if exhaustive:
        for plan in all_plans(kind, M, N, K):
            _evaluate(prob, plan, gate, seen)
    else:
        frontier = [t for t in (_evaluate(prob, normalise(kind, K, p), gate, seen) for p in start if valid(kind, M, N, K, p)) if t.correct]
        for _ in range(iterations):
            children: List[Trial] = []
            for parent in frontier:
                for plan in neighbours(kind, M, N, K, parent.plan):
                    fresh = plan not in seen
                    child = _evaluate(prob, plan, gate, seen)
                    # a child enters the beam only if it is correct and faster than the parent it came from
                    if fresh and child.correct and child.us < parent.us:
                        children.append(child)
            if not children:
                break
            frontier = sorted(frontier + children, key=lambda t: t.us)[:beam]
    good = [t for t in seen.values() if t.correct]
    if not good:
        raise RuntimeError("no candidate passed the correctness gate")
    finalists = sorted(good, key=lambda t: t.us)[:FINALISTS]
    for p in list(start)[:1]:  # the plan the search started from (the library's own) is always measured again
        own = seen.get(normalise(kind, K, p)) if valid(kind, M, N, K, p) else None
        if own is not None and own.correct and own not in finalists:
            finalists.append(own)
    if len(finalists) > 1:  # the quick ranking picks the finalists, a longer measurement of each decides
        for t in finalists:
            prob.run(t.plan)
            t.us = prob.confirm(lambda: prob.run(t.plan))
    best = min(finalists, key=lambda t: t.us)
    return TuneResult(best.plan, best.us, list(seen.values()))


def _workspace_pool(device):
    """workspace(nbytes) -> a device buffer of that size (None for 0), keeping only the latest one alive."""
    cache: Dict[int, torch.Tensor] = {}

    def workspace(nbytes: int):
        if nbytes == 0:
            return None
        if nbytes not in cache:
            cache.clear()
            cache[nbytes] = torch.empty(nbytes, dtype=torch.uint8, device=device)
        return cache[nbytes]

    return workspace


def _i8_problem(A, B, bias, C, shift: int, act: int) -> _Problem:
    M, K = A.shape
    N = B.shape[1]
    workspace = _workspace_pool(A.device)

    def run(plan: Plan):
        ws = workspace(ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, plan[0], plan[1]))
        ops.ac_gemm_i8_planned(A, B, bias, C, shift, act, plan[0], plan[1], workspace=ws)

    def reference():
        ops.ac_gemm_i8(A, B, bias, C, shift, act, workspace=workspace(ops.ac_gemm_i8_workspace_bytes(M, N, K)))

    return _Problem("i8", M, N, K, run, reference, C, exact=True)


def _bf16_problem(A, B, C, alpha: float, beta: float) -> _Problem:
    if beta != 0.0:
        raise ValueError("tune with beta == 0: the candidates overwrite C between runs")
    M, K = A.shape
    N = B.shape[1]
    workspace = _workspace_pool(A.device)

    def run(plan: Plan):  # K slices are summed through a workspace (same result on every run), not with atomics
        ws = workspace(ops.ac_gemm_bf16_planned_workspace_bytes(M, N, K, plan[0], plan[1]))
        ops.ac_gemm_bf16_planned(A, B, C, alpha, beta, plan[0], plan[1], workspace=ws)

    reference = lambda: ops.ac_gemm_bf16(A, B, C, alpha, beta)
    return _Problem("bf16", M, N, K, run, reference, C, exact=False)


def _conv_problem(x, w, bias, out, stride: int, pad: int, shift: int, act: int) -> _Problem:
    Nb, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    M, N, K = out.shape[0] * out.shape[1] * out.shape[2], Cout, KH * KW * Cin
    workspace = _workspace_pool(x.device)

    def run(plan: Plan):
        ws = workspace(ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, plan[0], plan[1]))
        ops.ac_conv2d_i8(x, w, bias, out, stride, pad, shift, act, workspace=ws, plan=plan)

    def reference():
        ops.ac_conv2d_i8(x, w, bias, out, stride, pad, shift, act, workspace=workspace(ops.ac_gemm_i8_workspace_bytes(M, N, K)))

    return _Problem("conv", M, N, K, run, reference, out, exact=True)


def tune_gemm_i8(A, B, bias, C, shift: int, act: int, gate=None, start: Optional[Iterable[Plan]] = None,
                 beam: int = 3, iterations: int = 4, exhaustive: bool = False) -> TuneResult:
    """Best (tile, splits) for this int8 GEMM.  `start`: plans to seed the beam with (default: seed_plans());
    pass the plan recorded for a related shape to reuse it.  `gate(C) -> bool` decides whether a
    candidate's output is correct.  C is overwritten."""
    prob = _i8_problem(A, B, bias, C, shift, act)
    seeds = list(start) if start is not None else seed_plans("i8", prob.M, prob.N, prob.K, ops.ac_gemm_i8_auto_plan(prob.M, prob.N, prob.K, True))
    return _search(prob, gate, seeds, beam, iterations, exhaustive)


def tune_gemm_bf16(A, B, C, alpha: float = 1.0, beta: float = 0.0, gate=None, start: Optional[Iterable[Plan]] = None,
                   beam: int = 3, iterations: int = 4, exhaustive: bool = False) -> TuneResult:
    """Best (tile, splits) for this bf16 GEMM; arguments as for tune_gemm_i8."""
    prob = _bf16_problem(A, B, C, alpha, beta)
    seeds = list(start) if start is not None else seed_plans("bf16", prob.M, prob.N, prob.K, ops.ac_gemm_bf16_auto_plan(prob.M, prob.N, prob.K))
    return _search(prob, gate, seeds, beam, iterations, exhaustive)


def tune_conv2d_i8(x, w, bias, out, stride: int, pad: int, shift: int, act: int, gate=None,
                   start: Optional[Iterable[Plan]] = None, beam: int = 3, iterations: int = 4, exhaustive: bool = False) -> TuneResult:
    """Best (kernel / tile, splits) for this NHWC int8 convolution: the tiled kernels with their K splits, the
    weight-stationary kernel and the patch kernel (codes 161 / 321), each where the geometry admits it.  Arguments
    as for tune_gemm_i8; `out` is overwritten."""
    prob = _conv_problem(x, w, bias, out, stride, pad, shift, act)
    seeds = list(start) if start is not None else seed_plans("conv", prob.M, prob.N, prob.K, ops.ac_gemm_i8_auto_plan(prob.M, prob.N, prob.K, True))
    return _search(prob, gate, seeds, beam, iterations, exhaustive)


class PlanBook:
    """Recorded best plans by (kind, M, N, K), with the lookup rule of the paper's schedule reuse: a new shape
    starts from the plan of a recorded shape with the same aspect ratio or with two dimensions in common."""

    def __init__(self):
        self.plans: Dict[Tuple[str, int, int, int], Plan] = {}

    def record(self, kind: str, M: int, N: int, K: int, plan: Plan) -> None:
        self.plans[(kind, M, N, K)] = (int(plan[0]), int(plan[1]))

    def related(self, kind: str, M: int, N: int, K: int) -> List[Plan]:
        out: List[Plan] = []
        for (k2, m, n, k), plan in self.plans.items():
            if k2 != kind:
                continue
            same_ratio = m * N == M * n and n * K == N * k
            shared = (m == M) + (n == N) + (k == K)
            if (same_ratio or shared >= 2) and plan not in out:
                out.append(plan)
        return out

    def save(self, path: str) -> None:
        with open(path, "w") as f:
            json.dump([[*key, *plan] for key, plan in sorted(self.plans.items())], f)

    @classmethod
    def load(cls, path: str) -> "PlanBook":
        book = cls()
        with open(path) as f:
            for kind, M, N, K, tile, splits in json.load(f):
                book.record(kind, M, N, K, (tile, splits))
        return book
