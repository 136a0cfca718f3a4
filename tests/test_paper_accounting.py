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
