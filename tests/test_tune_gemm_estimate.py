"""The tool that re-fits the GEMM's launch-time estimate: its copy of the estimate on hand-computed cases, and the fit
on timings generated from known constants (no GPU needed)."""
import random

from paper_2403_20041_amd import tune_gemm_estimate as tool


def test_estimate_by_hand():
    p = list(tool.START)
    # flat tile: a = 1.6 / 2.0 / 2.0 at fill just above 1/2, 3/4, 1; b = 4.4.  M = 128, N = 65536: 2 x 256 = 512 tiles of
    # 64 x 256 = one full round of K / 128 = 16 pairs
    assert abs(tool.estimate(p, 128, 65536, 2048, "f", 1) - (16 * 2.0 + 4.4)) < 1e-9
    # 256 of them (fill 1/2, a = 1.45), in two splits of 8 pairs: one full round again, plus the reduction of 2 slabs
    want = 8 * 2.0 + 4.4 + 4.9 + 0.18 * 2 * 128 * 32768 * 4 / 1e6
    assert abs(tool.estimate(p, 128, 32768, 2048, "f", 2) - want) < 1e-9
    assert abs(tool.estimate(p, 128, 32768, 2048, "f", 1) - (16 * 1.45 + 4.4)) < 1e-9
    # large tile, 300 tiles evenly scheduled: one whole round, 44 tiles shared out, 256 / 44 + 1 sharers per tile
    want = (16 * 3.5 + 9.3) + 44 * 16 / 256 * 3.5 + 9.3 + 35.0 + 0.7 * (256 / 44 + 1)
    assert abs(tool.estimate(p, 256 * 10, 256 * 30, 2048, "b", "sk") - want) < 1e-9


def test_fit_recovers_the_choices(tmp_path, capsys):
    rnd = random.Random(1)
    truth = [v * rnd.uniform(0.9, 1.1) for v in tool.START]
    path = tmp_path / "timings.txt"
    with open(path, "w") as f:
        for _ in range(40):
            M, N, K = rnd.randint(65, 4096), 128 * rnd.randint(8, 160), 128 * rnd.randint(8, 112)
            for tile, (bm, bn, cap, _) in tool.TILES.items():
                tiles = -(-M // bm) * -(-N // bn)
                for s in ((1,) if tiles >= tool.CU else (1, 2, 4)):
                    f.write("%d %d %d %s %s %.3f\n" % (M, N, K, tile, s, tool.estimate(truth, M, N, K, tile, s)))
            big = -(-M // 256) * -(-N // 256)
            if big >= 128 and big % tool.CU:
                f.write("%d %d %d b sk %.3f\n" % (M, N, K, tool.estimate(truth, M, N, K, "b", "sk")))
    groups = tool.read_timings([str(path)])
    assert len(groups) == 40
    tool.fit([str(path)])
    out = capsys.readouterr().out
    assert "geometric mean 1.00" in out and "kBigCost{{" in out and "kReduceUs" in out
