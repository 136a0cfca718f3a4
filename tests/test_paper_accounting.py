"""The benchmark's byte accounting and break-even formula against what the paper prints
(fixtures under tests/golden/, each citing its passage)."""
import os

import numpy as np

import bench
import kcache_inputs as ki

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_table1():
    rows = {}
    for line in open(os.path.join(GOLDEN, "table1_kcache_io.txt")):
        line = line.split("#")[0].strip()
        if line:
            name, flops, io = [x.strip() for x in line.split(";")]
            rows[name] = (flops, io)
    return rows


def read_eq4():
    vals = {}
    for line in open(os.path.join(GOLDEN, "eq4_breakeven.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = [x.strip() for x in line.split("=")]
            vals[k] = float(v)
    return vals


def test_algorithmic_bytes_are_the_dominant_terms_of_table_1():
    # multi-head attention in fp16, every sequence at full length: config 2 and config 5
    rows = read_table1()
    for cfg in (2, 5):
        wl = ki.config(cfg)
        env = dict(b=wl.B, n=wl.H, h=wl.d, d=wl.H * wl.d, s=wl.S_cap, N=wl.N)
        k_bytes, v_bytes = bench.algorithmic_bytes(wl, wl.seq_lens())
        io_s = [eval(t, {}, env) for t in rows["topn_softmax"][1].split("+")]
        io_a = [eval(t, {}, env) for t in rows["partial_v"][1].split("+")]
        assert k_bytes == io_s[1] == 2 * wl.B * wl.H * wl.d * wl.S_cap        # 2bnhs: the K rows
        assert v_bytes == io_a[1] == 2 * wl.B * wl.N * wl.H * wl.d            # 2bNd: the V rows
        # everything else in those two rows (q, positions / weights, output) is below 1 %
        rest = io_s[0] + io_s[2] + io_a[0] + io_a[2]
        assert rest < 0.01 * (k_bytes + v_bytes)
        # the conventional cache moves s rows of V instead of N: the 2bsd term
        io_sv = [eval(t, {}, env) for t in rows["sv"][1].split("+")]
        assert io_sv[1] == k_bytes


def test_grouped_queries_and_ragged_lengths_in_the_accounting():
    wl = ki.config(3)                      # 32 query heads over 8 KV heads
    k_bytes, v_bytes = bench.algorithmic_bytes(wl, wl.seq_lens())
    assert k_bytes == wl.B * wl.Hkv * wl.S_cap * 256      # K rows are shared by a group
    assert v_bytes == wl.B * wl.H * wl.N * 256            # every query head pulls its own rows
    wl4 = ki.config(4)
    lens = wl4.seq_lens()
    k_bytes, v_bytes = bench.algorithmic_bytes(wl4, lens)
    assert k_bytes == int(lens.astype(np.int64).sum()) * wl4.Hkv * 256
    short = np.array([5, 1000], dtype=np.int32)
    assert bench.algorithmic_bytes(wl4.replace(B=2), short)[1] == (5 + wl4.N) * wl4.H * 256
    assert bench.algorithmic_bytes(wl, wl.seq_lens(), k_elem_bytes=1)[0] * 2 == \
        bench.algorithmic_bytes(wl, wl.seq_lens())[0]


def test_break_even_formula_reproduces_the_papers_a100_example():
    g = read_eq4()
    r = bench.eq4_break_even(g["bandwidth_gpu_GBps"], g["bandwidth_h2d_GBps"])
    assert round(r) == g["threshold_s_over_N"]
    assert bench.eq4_break_even(g["bandwidth_gpu_GBps"], g["bandwidth_h2d_GBps"],
                                overlapped=True) == r / 2


def test_break_even_for_groups_follows_from_the_byte_counts():
    # with G query heads per KV head the launch floors of the accounting cross at G times the
    # single-head ratio: K and V of a position are read from HBM once per group, the N rows of
    # V cross the link once per query head
    hbm, link = 7000.0, 55.0
    for G in (1, 4, 8):
        wl = ki.config(3).replace(H=8 * G, Hkv=8, B=4, S_cap=1 << 20, len_range=None)
        N = 64
        ratio = bench.eq4_break_even(hbm, link, overlapped=True, G=G)
        for s, kcache_wins in ((int(0.9 * ratio * N), False), (int(1.1 * ratio * N), True)):
            lens = np.full(wl.B, s, dtype=np.int32)
            k_bytes, v_bytes = bench.algorithmic_bytes(wl, lens, N=N)
            t_kcache = max(k_bytes / hbm, v_bytes / link)      # the two transfers overlap
            t_conventional = 2 * k_bytes / hbm                  # K and V rows from HBM
            assert (t_kcache <= t_conventional) == kcache_wins, (G, s)


def read_sweep():
    """Rows of the tracked config-4 sweep (profiles/config4_sweep.md): measured on the MI355X."""
    path = os.path.join(os.path.dirname(GOLDEN), "..", "profiles", "config4_sweep.md")
    rows = []
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 8 and cells[1].isdigit():
            rows.append(dict(frac=float(cells[0]), N=int(cells[1]), us=float(cells[2]),
                             tps=float(cells[3]), floor=float(cells[6]), bound=cells[7]))
    return rows


def test_launch_floor_model_follows_table_1_and_equation_3():
    # K term independent of N, V term proportional to N; the floor is the larger of the two
    # (equation (3) read with overlapped transfers), so it never falls as N grows and grows in
    # proportion to N once the V rows bind.
    wl = ki.config(4)
    lens = wl.seq_lens()
    floors = [bench.launch_floor_us(wl, lens, N, 8000.0, 57.2) for N in bench.SWEEP_N]
    assert all(abs(f[1] - floors[0][1]) < 1e-9 for f in floors)            # K time: no N in it
    assert all(b[0] >= a[0] for a, b in zip(floors, floors[1:]))
    for (a, N0), (b, N1) in zip(zip(floors, bench.SWEEP_N), zip(floors[1:], bench.SWEEP_N[1:])):
        assert abs(b[2] / a[2] - N1 / N0) < 1e-9                            # V time: linear in N
    link_bound = [f for f in floors if f[2] > f[1]]
    assert len(link_bound) >= 3 and all(f[0] == f[2] for f in link_bound)


def test_measured_sweep_shows_the_trend_of_table_4():
    # Table 4 of the paper: at a fixed shape throughput does not rise with N.  The tracked
    # measurement must show the same, stay above the floor of the accounting everywhere, and
    # scale with N where the host link binds.
    rows = read_sweep()
    assert len(rows) == len(bench.SWEEP_N) * len(bench.SWEEP_FRAC)
    wl = ki.config(4)
    lens = wl.seq_lens()
    for frac in bench.SWEEP_FRAC:
        cells = sorted((r for r in rows if r["frac"] == frac), key=lambda r: r["N"])
        assert [c["N"] for c in cells] == list(bench.SWEEP_N)
        for a, b in zip(cells, cells[1:]):
            # flat (within 5 %) while the K scan binds, falling once the V rows do
            assert b["tps"] <= a["tps"] * 1.05, "throughput rises with N at fraction %g" % frac
        for c in cells:
            floor, t_hbm, t_link = bench.launch_floor_us(wl, lens, c["N"], 8000.0, 57.2)
            assert abs(floor - c["floor"]) / floor < 0.01          # the table's own floor column
            assert c["us"] >= floor                                  # nothing beats the floor
            assert c["bound"] == ("hbm" if t_hbm >= t_link else "host_link")
            if t_link > 1.5 * t_hbm:                                 # clearly link bound
                assert c["us"] <= 1.15 * floor
        by_n = {c["N"]: c["us"] for c in cells}
        assert abs(by_n[512] / by_n[256] - 2.0) < 0.2               # proportional to N
        assert cells[-1]["tps"] < 0.25 * cells[0]["tps"]


def test_bench_refuses_more_than_one_gpu():
    # the bench contract of this build: one GPU; a request for more exits with a message
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr + r.stdout
    assert not r.stdout.strip().startswith("{")
