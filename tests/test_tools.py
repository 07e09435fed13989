"""Host-side tools around the library: the table report and the strategy-study helpers."""
import io
import contextlib

from paper_1703_06503_amd import report


def test_report_reads_old_and_new_tables(tmp_path):
    t = tmp_path / "table.txt"
    t.write_text("# M N K layout ms MWG NWG KWG MDIMC NDIMC VWM VWN SA SB PAD KWI MFMA GRP SK NS\n"
                 "4096 4096 4096 0 1.0 256 256 32 16 16 4 4 1 1 1 8 1 0 1 2\n"
                 "1024 1024 1024 0 0.05 128 128 16 16 16 4 4 1 1 1 8 1 1\n"          # no SK, NS
                 "128 4096 4096 1 0.05 64 128 32 16 16 4 4 1 1 0 2 1 1 8 2\n"
                 "garbage line\n")
    rows = report.read_table(str(t))
    assert len(rows) == 3
    assert rows[1][5] == [128, 128, 16, 16, 16, 4, 4, 1, 1, 1, 8, 1, 1, 1, 2, 1]
    out = io.StringIO()
    with contextlib.redirect_stdout(out):
        assert report.main([str(t), "--peak-tflops", "157.3"]) == 0
    text = out.getvalue()
    # 2 * 4096^3 flop in 1 ms = 137 439 GFLOP/s = 87.4 % of 157.3 TFLOP/s
    assert "| 137439 | 87.4 |" in text
    assert text.count("\n") == 2 + 3


def test_convolution_figures_of_merit_are_the_papers_counts():
    """GFLOP/s = (1 + 2 Xf Yf) X Y / t and GB/s = 2 X Y floats / t (footnote of the section
    "Best-found results" of the convolution case study)."""
    from paper_1703_06503_amd import conv_cli, synth
    w = synth.CONV_WORKLOADS["conv_7x7"]
    gf, gb = conv_cli.figures(w, 1.0)                      # one millisecond
    assert gf == (1 + 2 * 49) * 8192 * 4096 / 1e6 and gb == 2 * 8192 * 4096 * 4 / 1e6
    assert synth.make_conv_inputs(8, 4, 3, 3, seed=1)[0].shape == (6, 10)


def test_strategy_study_accepts_the_convolution_spaces():
    import numpy as np
    from paper_1703_06503_amd import strategy_study as ss
    n, replay = ss.space_size_and_replay("conv7x7")
    table = np.linspace(1.0, 2.0, n).astype(np.float32)     # configuration 0 is the optimum
    opt, rows = ss.study(table, replay, 20, 4)
    assert opt == 1.0 and len(rows) == 6
    assert all(0 < r["mean_pct_of_best"] <= 100.0 for r in rows)


def test_recorded_full_searches_cover_their_spaces():
    """The committed tables of the two recorded GEMM full searches hold one row per
    configuration of the space they name, and the optimum that the studies are measured against
    is the configuration their write-ups name."""
    import os
    import numpy as np
    from paper_1703_06503_amd import binding as b
    from paper_1703_06503_amd import strategy_study as ss
    results = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "results")
    for name, space, tile in [("full_search_cfg2_2048.csv", "full", (128, 64, 32)),
                              ("full_search_cfg4_4096_mfma.csv", "mfma", (256, 256, 32))]:
        n, _ = ss.space_size_and_replay(space)
        with open(os.path.join(results, name)) as f:
            assert sum(1 for _ in f) == n + 1                       # header + one row each
        table = ss.load_table(os.path.join(results, name), n)
        timed = table > 0
        assert timed.sum() >= 0.99 * n                              # the rest spilled registers
        best = b.sgemm_space_get(ss.SPACES[space], int(np.argmin(np.where(timed, table, np.inf))))
        assert (best.mwg, best.nwg, best.kwg) == tile
