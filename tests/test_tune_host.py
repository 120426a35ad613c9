"""Host logic of the plan search: candidate enumeration, the beam rule and schedule reuse (no device needed)."""
import torch

from paper_2505_18574_amd import tune


def test_k_tiles_and_normalise():
    assert tune.k_tiles("i8", 4096, 64) == 32 and tune.k_tiles("i8", 4096, 256) == 64
    assert tune.k_tiles("bf16", 4096, 128) == 64 and tune.k_tiles("bf16", 4100, 256) == 129
    # 32 K tiles over 12 slices: 3 tiles each, so only 11 slices hold work
    assert tune.normalise("i8", 4096, (64, 12)) == (64, 11)
    assert tune.normalise("i8", 4096, (64, 1)) == (64, 1)
    assert tune.normalise("i8", 64, (256, 8)) == (256, 1)


def test_all_plans_and_neighbours():
    plans = tune.all_plans("i8", 128, 1024, 1024)
    assert (64, 1) in plans and (128, 8) in plans and (192, 8) in plans and (256, 16) in plans
    assert all(tune.valid("i8", 128, 1024, 1024, p) for p in plans)
    assert (64, 16) not in plans  # 1024 bytes of K are 8 tiles of 128 bytes
    assert len(set(plans)) == len(plans)
    nb = tune.neighbours("i8", 128, 1024, 1024, (128, 2))
    assert set(nb) == {(64, 2), (192, 2), (128, 1), (128, 4)}
    assert tune.neighbours("bf16", 4096, 4096, 16, (256, 1)) == [(192, 1)]  # one K tile: nothing to split
    # a split that would need more than the workspace cap is not offered
    assert not tune.valid("i8", 16384, 16384, 4096, (64, 2))


def test_seed_plans_cover_every_tile():
    # one 256 x 256 output tile with a very deep K: each tile size starts from the split that fills 256 CUs
    seeds = tune.seed_plans("bf16", 256, 256, 524288, (64, 16))
    assert seeds == [(64, 16), (128, 64), (192, 128), (256, 256)]
    # a shape with plenty of tiles starts unsplit on every tile size; the library's plan comes first, once
    assert tune.seed_plans("i8", 4096, 4096, 4096, (256, 1)) == [(256, 1), (64, 1), (128, 1), (192, 1)]
    # splits never exceed the K tiles of the tile's kernel
    # ... and a K short enough to stay resident also starts on the weight-stationary tiles
    assert tune.seed_plans("i8", 64, 64, 256, (64, 1)) == [(64, 1), (64, 2), (128, 2), (192, 2), (256, 4), (160, 1), (320, 1)]
    assert tune.valid("i8", 4096, 64, 1536, (320, 1)) and not tune.valid("i8", 4096, 64, 1537, (320, 1))
    assert tune.valid("i8", 4096, 64, 2048, (160, 1)) and not tune.valid("i8", 4096, 64, 512, (160, 2))
    assert not tune.valid("bf16", 4096, 64, 512, (320, 1))
    assert set(tune.neighbours("i8", 4096, 64, 512, (320, 1))) == {(160, 1), (64, 1), (192, 1)}


def test_convolution_plan_space():
    # a convolution adds the patch kernel's two unit sizes to the int8 plan space; they never split K
    M, N, K = 8 * 56 * 56, 64, 576
    plans = tune.all_plans("conv", M, N, K)
    assert set(tune.all_plans("i8", M, N, K)) | {(161, 1), (321, 1)} == set(plans)
    assert tune.valid("i8", M, N, K, (32, 1)) and tune.valid("conv", M, N, K, (32, 1)) and not tune.valid("bf16", M, N, K, (32, 1))
    assert tune.valid("i8", M, N, K, (32, 2)) and not tune.valid("i8", M, N, K, (32, 10))  # K slices of whole 64-byte tiles: nine here
    assert not tune.valid("i8", M, N, 600, (32, 1)) and not tune.valid("i8", M, N, 32, (32, 1))
    assert (32, 1) in tune.neighbours("i8", M, N, K, (64, 1)) and set(tune.neighbours("i8", M, N, K, (32, 1))) == {(64, 1), (32, 2)}
    assert set(tune.neighbours("i8", M, N, K, (32, 2))) == {(64, 2), (32, 1), (32, 3)}  # four slices of nine K tiles are three
    assert tune.valid("conv", M, N, K, (321, 1)) and not tune.valid("conv", M, N, K, (321, 2))
    assert not tune.valid("i8", M, N, K, (321, 1)) and not tune.valid("bf16", M, N, K, (161, 1))
    seeds = tune.seed_plans("conv", M, N, K, (64, 1))
    assert seeds[0] == (64, 1) and {(160, 1), (320, 1), (161, 1), (321, 1)} <= set(seeds)
    assert set(tune.neighbours("conv", M, N, K, (321, 1))) == {(161, 1), (160, 1), (320, 1), (64, 1), (192, 1)}
    assert {(161, 1), (321, 1)} <= set(tune.neighbours("conv", M, N, K, (320, 1)))
    assert tune.k_tiles("conv", K, 64) == tune.k_tiles("i8", K, 64)


class FakeProblem(tune._Problem):
    """A cost model in place of the device: latency by plan, and a set of plans whose output is 'wrong'."""

    def __init__(self, cost, wrong=()):
        self.launched = []
        out = torch.zeros(1)

        def run(plan):
            self.launched.append(plan)
            out[0] = -1.0 if plan in wrong else 1.0

        super().__init__("i8", 128, 1024, 1024, run, lambda: out.fill_(1.0), out, exact=True,
                         sync=lambda: None, measure=lambda fn: cost(self.launched[-1]))


def test_beam_keeps_correct_and_faster_candidates_only():
    cost = lambda p: {32: 45.0, 64: 30.0, 128: 20.0, 192: 35.0, 256: 40.0, 160: 50.0, 320: 60.0}[p[0]] / (1 + 0.5 * (p[1] > 1)) + p[1]
    # (128, 2) would be the fastest plan but produces a wrong result: it must never be chosen
    prob = FakeProblem(cost, wrong={(128, 2)})
    res = tune._search(prob, None, [(64, 1)], beam=2, iterations=6, exhaustive=False)
    assert res.best != (128, 2)
    assert {t.plan: t.correct for t in res.trials}[(128, 2)] is False
    want = min((p for p in tune.all_plans("i8", 128, 1024, 1024) if p != (128, 2)), key=cost)
    full = tune._search(FakeProblem(cost, wrong={(128, 2)}), None, [], 1, 0, exhaustive=True)
    assert full.best == want and abs(full.best_us - cost(want)) < 1e-9
    assert res.best_us <= cost((64, 1))  # the beam never ends worse than its seed


def test_finalists_are_measured_again_before_the_best_is_named():
    """The quick measurement ranks (here: with an error that favours a slower plan); the three best by it are
    measured again with the longer one, which decides."""
    true = lambda p: 10.0 + abs(p[0] - 128) / 16.0 + p[1]
    quick = lambda p: true(p) - (5.0 if p == (64, 1) else 0.0)  # the quick look flatters (64, 1)
    prob = FakeProblem(quick)
    prob.confirm = lambda fn: true(prob.launched[-1])
    res = tune._search(prob, None, [], 1, 0, exhaustive=True)
    assert quick((64, 1)) < quick((128, 1)) and res.best == (128, 1) and res.best_us == true((128, 1))
    by_plan = {t.plan: t.us for t in res.trials}
    assert by_plan[(64, 1)] == true((64, 1))          # a finalist: carries the longer measurement
    assert by_plan[(256, 1)] == quick((256, 1))       # not a finalist: the quick one
    # the plan a beam search starts from is measured again even when the quick look ranks it last
    quick2 = lambda p: true(p) + (100.0 if p == (128, 1) else 0.0)
    prob = FakeProblem(quick2)
    prob.confirm = lambda fn: true(prob.launched[-1])
    res = tune._search(prob, None, [(128, 1)], beam=3, iterations=2, exhaustive=False)
    assert res.best == (128, 1) and res.best_us == true((128, 1))


def test_beam_stops_when_no_child_improves():
    prob = FakeProblem(lambda p: 10.0 + abs(p[0] - 128) + p[1])  # (128, 1) is a strict local and global minimum
    res = tune._search(prob, None, [(128, 1)], beam=3, iterations=5, exhaustive=False)
    assert res.best == (128, 1)
    assert len(res.trials) == 1 + len(tune.neighbours("i8", 128, 1024, 1024, (128, 1)))


def test_plan_book_reuse_rule(tmp_path):
    book = tune.PlanBook()
    book.record("i8", 1024, 1024, 1024, (128, 1))
    book.record("i8", 12544, 64, 256, (64, 1))
    book.record("bf16", 512, 512, 512, (64, 2))
    assert book.related("i8", 512, 512, 512) == [(128, 1)]        # same aspect ratio
    assert book.related("i8", 6272, 64, 256) == [(64, 1)]         # two dimensions in common
    assert book.related("i8", 6272, 128, 64) == []
    assert book.related("bf16", 1024, 1024, 1024) == [(64, 2)]
    path = str(tmp_path / "plans.json")
    book.save(path)
    assert tune.PlanBook.load(path).plans == book.plans


def test_tile_tables_agree_with_the_library():
    """tune.py restates the library's tile codes, K-tile depths and residency limits on the host side: every code,
    over a sweep of K and split counts, is checked against what the planned entry points accept (empty problems,
    so nothing is launched and no pointer is read) and against the workspace they ask for."""
    from paper_2505_18574_amd import ops

    L = ops.lib()
    codes = list(tune.TILES) + list(tune.WS_TILES) + list(tune.HALO_TILES) + [0, 32, 96, 255, 512]
    for kind in ("i8", "bf16"):
        for tile in codes:
            for K in (16, 64, 128, 640, 1024, 1536, 1552, 2048, 2064, 4096, 8192 + 16):
                for splits in (1, 2, 3, 8, 16, 33, 64, 65, 1000):
                    if kind == "i8":
                        st = L.ac_gemm_i8_planned(None, K, None, 64, None, 0, None, 64, 0, 64, K, 8, 0, None, 0, tile, splits, None)
                    else:
                        st = L.ac_gemm_bf16_planned(None, K, None, 64, None, 64, 0, 64, K, 1.0, 0.0, None, 0, tile, splits, None)
                    # on an empty problem only the plan itself can be refused; the patch kernel is a convolution kernel
                    want = tune.valid(kind, 0, 64, K, (tile, splits))
                    assert (st == ops.AC_OK) == want, (kind, tile, K, splits, st)
                    assert st in (ops.AC_OK, ops.AC_ERR_PLAN)
                    if want and tile in tune.TILES:
                        t, s = tune.normalise(kind, K, (tile, splits))
                        M, N = 192, 128
                        fn = ops.ac_gemm_i8_planned_workspace_bytes if kind == "i8" else ops.ac_gemm_bf16_planned_workspace_bytes
                        assert fn(M, N, K, tile, splits) == (s * M * N * 4 if s > 1 else 0), (kind, tile, K, splits)
    # the convolution entry point takes the patch-kernel codes and refuses a K split of them
    for tile in tune.HALO_TILES:
        assert L.ac_conv2d_i8_planned(None, None, None, None, 0, 56, 56, 64, 64, 3, 3, 1, 1, 9, 1, None, 0, tile, 1, None) == ops.AC_OK
        assert L.ac_conv2d_i8_planned(None, None, None, None, 0, 56, 56, 64, 64, 3, 3, 1, 1, 9, 1, None, 0, tile, 2, None) == ops.AC_ERR_PLAN
