"""CPU-only checks of the boundary: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2308_01320_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "he.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(he_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS), names
    for n in names:
        assert getattr(L, n) is not None


def test_workspace_bytes_is_pure_and_monotone():
    L = binding.lib()
    d = synth.CONFIGS["tiny"]
    c1 = binding.make_config(d)
    c2 = binding.make_config(d, max_batch=8)
    b1, b2 = L.he_workspace_bytes(C.byref(c1)), L.he_workspace_bytes(C.byref(c2))
    assert 0 < b1 < b2
    bad = binding.make_config(d)
    bad.hidden = 250  # not a multiple of n_heads
    assert L.he_workspace_bytes(C.byref(bad)) == 0
    assert L.he_workspace_bytes(None) == 0
    big = binding.make_config(synth.CONFIGS["opt-13b"])
    kv = 2 * 40 * 32 * 512 * 5120 * 2
    assert L.he_workspace_bytes(C.byref(big)) > kv  # at least the KV arena of the headline workload


def test_host_side_argument_errors_need_no_gpu():
    L = binding.lib()
    h = C.c_void_p()
    assert L.he_create(None, None, C.byref(h)) == 1
    assert b"NULL" in L.he_last_error(None)
    cfg = binding.make_config(synth.CONFIGS["tiny"])
    cfg.dtype = 7
    assert L.he_create(C.byref(cfg), None, C.byref(h)) == 1
    cfg = binding.make_config(synth.CONFIGS["tiny"])
    cfg.hidden = 250
    assert L.he_create(C.byref(cfg), None, C.byref(h)) == 2
    cfg = binding.make_config(synth.CONFIGS["tiny"])
    assert L.he_create(C.byref(cfg), None, C.byref(h)) == 1  # weights NULL
    assert L.he_destroy(None) == 0
    assert L.he_reset(None) == 1
    assert L.he_cache_len(None) == -1
    assert L.he_rng_words(0, 0, 0, 0, 4, None, None) == 1


def test_decode_gemm_plans_fit_the_chip_and_the_scratch():
    """Host logic of the launch planner: every plan puts at most one workgroup on a CU, leaves every
    wavefront at least 8 k-blocks, stays inside the k-split scratch, and is never worse balanced than
    32-row tiles alone."""
    import math
    cus = 256
    for name in ("opt-1.3b", "opt-6.7b", "opt-13b", "opt-66b"):
        d = synth.CONFIGS[name]
        H, F = d.hidden, d.ffn
        cap = 2 * 8 * 32 * H  # the engine's scratch for batches up to 32
        for (N, K, store) in ((3 * H, H, False), (F, H, False), (H, H, True), (H, F, True)):
            unit, per_wg, ks = binding.he_plan_decode_gemm(32, N, K, store, cap if store else 0, cus)
            assert unit in (16, 32) and per_wg >= 1 and 1 <= ks <= 8
            groups = math.ceil(N // unit / per_wg)
            assert groups * ks <= cus, (name, N, K, unit, per_wg, ks)
            assert (K // 16) // (ks * 4) >= 8 or ks == 1
            if not store:
                assert ks == 1
                assert unit * per_wg <= 32 * math.ceil(N // 32 / cus)  # the most loaded workgroup
            else:
                assert groups * ks * (2 * per_wg + 7) * 256 <= cap or unit == 32
    # 33..64 rows: two 32-row slices per workgroup, which only the 16-row-unit kernel takes, at most 8 units
    for (N, K, store) in ((3 * 5120, 5120, False), (20480, 5120, False), (5120, 5120, True), (5120, 20480, True)):
        unit, per_wg, ks = binding.he_plan_decode_gemm(64, N, K, store, 2 * 8 * 64 * 5120 if store else 0, 256)
        assert unit == 16 and 2 <= per_wg <= 8 and math.ceil(N // 16 / per_wg) * ks <= 256, (N, K, unit, per_wg, ks)
    # the case the 16-row units exist for: 640 tiles do not divide over 256 CUs, 1280 units do
    assert binding.he_plan_decode_gemm(32, 20480, 5120, False, 0, 256) == (16, 5, 1)
    assert binding.he_plan_decode_gemm(32, 15360, 5120, False, 0, 256) == (32, 2, 1)
    # fewer CUs, bigger shares: 640 tiles over 128 CUs are five each (nothing to gain from halves),
    # over 200 CUs four tiles (128 rows) or seven halves (112 rows)
    assert binding.he_plan_decode_gemm(32, 20480, 5120, False, 0, 128) == (32, 5, 1)
    assert binding.he_plan_decode_gemm(32, 20480, 5120, False, 0, 200) == (16, 7, 1)
    # at most 16 rows: the 16-row-unit kernel leaves out the unused half of the activation panel, so it wins
    # ties with the 32-row tiles (6.7B-shaped FC1: four units = two tiles), and the general checks still hold
    assert binding.he_plan_decode_gemm(16, 16384, 4096, False, 0, 256) == (16, 4, 1)
    assert binding.he_plan_decode_gemm(32, 16384, 4096, False, 0, 256) == (32, 2, 1)
    for M in (1, 8, 16):
        for (H, F) in ((2048, 8192), (4096, 16384), (5120, 20480), (9216, 36864)):
            for (N, K, store) in ((3 * H, H, False), (F, H, False), (H, H, True), (H, F, True)):
                unit, per_wg, ks = binding.he_plan_decode_gemm(M, N, K, store, 2 * 8 * 32 * H if store else 0, 256)
                assert math.ceil(N // unit / per_wg) * ks <= 256 and ((K // 16) // (ks * 4) >= 8 or ks == 1)
    with pytest.raises(binding.HeError):
        binding.he_plan_decode_gemm(32, 100, 64)


def test_prompt_gemm_plans_fill_the_chip_in_whole_rounds():
    """Host logic of the prompt-pass tile planner: tiles come in rounds of one per CU and a partly empty round costs a
    full one, so the plan picks the tile width (256 or 320 columns) and, for the GEMMs whose partial sums a LayerNorm
    adds, the columns to cut along k so that the rounds come out even."""
    import math
    # OPT-13B layer shape, batch 32 x prompt 256 = 8192 rows, 256 CUs: 320-column tiles divide everything
    assert binding.he_plan_prompt_gemm(8192, 15360, 5120) == (320, 1, 0)            # QKV: 48 x 32 tiles = six rounds
    assert binding.he_plan_prompt_gemm(8192, 20480, 5120) == (320, 1, 0)            # FC1: eight rounds
    assert binding.he_plan_prompt_gemm(8192, 5120, 5120, True) == (320, 1, 0)       # out-projection: two rounds, no cut
    assert binding.he_plan_prompt_gemm(8192, 5120, 20480, True) == (320, 1, 0)
    # ... and the scoring pass over 16384 rows
    assert binding.he_plan_prompt_gemm(16384, 5120, 20480, True) == (320, 1, 0)
    # hidden size 4096 (16 x 256 prompt rows): 256-column tiles fill whole rounds as they are
    assert binding.he_plan_prompt_gemm(4096, 12288, 4096) == (256, 1, 0)
    assert binding.he_plan_prompt_gemm(4096, 4096, 4096, True) == (256, 1, 0)
    # OPT-66B layer shape, 8 x 256 rows: 29 x 8 = 232 tiles of 320 columns are one round (288 of 256 columns: two)
    assert binding.he_plan_prompt_gemm(2048, 9216, 9216, True) == (320, 1, 0)
    # the same width with 32 x 256 rows: 36 x 32 = 1152 tiles of 256 columns; the last four columns of tiles are cut
    # in two (four rounds of whole tiles, then 256 half tiles); without scratch for a second set of sums nothing can
    # be cut, and 320-column tiles (928: four rounds) are the better of the whole-tile plans
    assert binding.he_plan_prompt_gemm(8192, 9216, 9216, True) == (256, 2, 8192)
    assert binding.he_plan_prompt_gemm(8192, 9216, 9216, True, 8192 * 9216) == (320, 1, 0)
    assert binding.he_plan_prompt_gemm(8192, 9216, 9216, False) == (320, 1, 0)
    # too few rows or tiles for the big tiles
    assert binding.he_plan_prompt_gemm(512, 5120, 5120)[0] == 0
    # general: whatever is picked, the whole tiles and the cut ones cover every column exactly once
    for M in (1024, 2048, 4096, 8192, 16384):
        for (N, K) in ((6144, 2048), (2048, 8192), (12288, 4096), (16384, 4096), (15360, 5120), (5120, 20480), (27648, 9216)):
            for cus in (64, 256, 304):
                cols, ks, split = binding.he_plan_prompt_gemm(M, N, K, True, 0, cus)
                if cols == 0:
                    continue
                assert cols in (256, 320) and ks in (1, 2) and 0 <= split < cols * math.ceil(N / cols)
                assert split % cols == 0 and (ks == 2 or split == 0), (M, N, K, cus, cols, ks, split)
    with pytest.raises(binding.HeError):
        binding.he_plan_prompt_gemm(8192, 100, 64)


def test_ksplit_hand_off_stays_inside_what_he_create_reserves():
    """The invariant the k-split hand-off of the decode out-projection / FC2 rests on.  Partial sums cross
    workgroups inside one launch through scratch, every (column group, row slice, split) in words of its own, with
    one arrival counter per (column group, row slice).  The account comes from the launcher's own choice of kernel
    variant and grid (a dry run of the launch, no device), so an index formula that outgrows the reserve shows here
    and not as a stray write on the GPU.  Checked: the words indexed fit the engine's scratch and the static
    entry point's share of its array; the counters and the column-group statistics fit their reserves -- for
    every model shape of the benchmark configurations and a set of narrow ones, 16-bit and 8-bit weights, every
    batch up to 64 and three chip sizes."""
    import dataclasses
    shapes = [synth.CONFIGS[n] for n in synth.CONFIGS]
    for H, nh, F in ((64, 1, 64), (64, 1, 256), (128, 2, 512), (192, 3, 768), (256, 2, 1024), (512, 4, 2048),
                     (1024, 8, 4096)):
        shapes.append(dataclasses.replace(synth.CONFIGS["tiny"], hidden=H, n_heads=nh, ffn=F))
    seen_split = False
    for d in shapes:
        d = dataclasses.replace(d, dtype="bf16")
        for fp8 in (0, 1):
            for max_batch in (1, 16, 32, 64):
                cfg = binding.make_config(d, max_batch=max_batch, max_seq_len=64, weights_fp8=fp8)
                for B in sorted({1, 8, 16, 17, 32, 33, 48, 49, 64, max_batch}):
                    if B > max_batch or (fp8 and B > 32):
                        continue
                    for which in (0, 1):
                        for cus in (64, 256, 304):
                            a = binding.he_decode_scratch_account(cfg, B, which, cus)
                            case = (d.hidden, d.ffn, fp8, max_batch, B, which, cus)
                            assert 1 <= a.ksplit <= 8, case
                            assert a.scratch_floats <= a.scratch_reserved, case
                            assert a.scratch_floats <= a.static_floats, case
                            assert a.counters <= a.counters_reserved, case
                            assert a.stat_pairs <= a.stat_pairs_reserved, case
                            # (column group, row slice, split) regions are equal runs laid end to end: whole
                            # numbers of 256-float wavefront rows, so no two of them share a word
                            if a.ksplit > 1:
                                seen_split = True
                                assert a.scratch_floats % (a.counters * a.ksplit * 256) == 0, case
    assert seen_split
    d = dataclasses.replace(synth.CONFIGS["tiny"], dtype="bf16")
    with pytest.raises(binding.HeError):
        binding.he_decode_scratch_account(binding.make_config(d, max_batch=8, max_seq_len=64), 9, 0, 256)
    with pytest.raises(binding.HeError):
        binding.he_decode_scratch_account(binding.make_config(dataclasses.replace(d, dtype="f32"), max_batch=8,
                                                              max_seq_len=64), 8, 0, 256)


def test_bench_clock_sampler_reads_the_marked_level(tmp_path):
    """bench.py's clock record: the level the driver marks with '*' in its text files, sampled from a thread."""
    import importlib.util
    import time
    spec = importlib.util.spec_from_file_location("bench", os.path.join(os.path.dirname(__file__), "..", "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    (tmp_path / "sclk").write_text("0: 132Mhz\n1: 500Mhz\n2: 2400Mhz *\n")
    (tmp_path / "mclk").write_text("0: 900Mhz\n1: 2000Mhz *\n")
    (tmp_path / "level").write_text("auto\n")
    c = bench.ClockSampler(period_s=0.005)
    c.files = {"sclk": str(tmp_path / "sclk"), "mclk": str(tmp_path / "mclk"), "level": str(tmp_path / "level")}
    c.start()
    time.sleep(0.03)
    c.finish()
    rec = c.record()
    assert rec["sclk_mhz"]["min"] == rec["sclk_mhz"]["max"] == 2400 and rec["sclk_mhz"]["samples"] >= 1
    assert rec["mclk_mhz"]["median"] == 2000 and rec["performance_level"] == "auto"
    # no driver files (as on a box without the GPU): the record says so instead of failing
    d = bench.ClockSampler()
    d.files = {}
    d.start()
    d.finish()
    assert d.record()["sclk_mhz"] is None
