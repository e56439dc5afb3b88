"""No-GPU checks of the benchmark's host logic: the algorithmic byte / operation counts behind the roofline
entries, for every workload shape, against counts written out by hand."""
import bench
import workloads as wl


def test_every_workload_has_a_roofline_entry_for_each_kernel_class():
    classes = ["ks_pre", "ks_modup_fcols", "ks_frows", "ks_inner_irows", "ks_inner_irows_wide", "ks_icols_special",
               "ks_icols_moddown", "byte_planes", "pm_fcols", "pm_frows_mac_irows", "pm_icols_last", "pm_icols_rescale"]
    for w in wl.WORKLOADS:
        if w.log_n != 16:
            continue
        for c in classes:
            dom, roof = bench.roofline_for(w, {c: (1.0, 1)})
            assert dom == c and roof["bound"] == "hbm" and roof["peak"] == 8000.0
            assert roof["achieved"] >= 0.0 and abs(roof["frac"] - roof["achieved"] / 8000.0) < 1e-12


def test_key_switch_counts_of_the_microbenchmark():
    w = wl.BY_NAME["keyswitch"]  # 64 rotations, L = 10, K = 3, alpha = 3 -> beta = 4, ext = 13
    unit = 8.0 * w.N
    _, roof = bench.roofline_for(w, {"ks_frows": (1.0, 1)})
    assert abs(roof["achieved"] - 64 * 2 * (4 * 13 + 10) * unit / 1e-3 / 1e9) < 1e-6  # digits and P*c0 in and out
    _, roof = bench.roofline_for(w, {"ks_inner_irows": (2.0, 1)})
    units = 64 * (4 * 10 + 10 + 2 * 10) + 64 * 2 * 4 * 10  # digits, P*c0, accumulators; one key per rotation
    assert abs(roof["achieved"] - units * unit / 2e-3 / 1e9) < 1e-6
    assert bench.stagewise_rotation_units(w) == 486


def test_matrix_core_operation_count():
    w = wl.BY_NAME["ffn2560"]
    _, roof = bench.roofline_for(w, {"accumulate_mfma": (100.0, 9)})
    # outputs x operands x limb words x byte planes; the second layer runs after the rescale, at 15 limbs
    ops = 2.0 * (2560 * 6912 * 2 * 16 + 6912 * 2560 * 2 * 15) * 65536 * 7
    assert roof["bound"] == "mfma" and roof["peak"] == 5000.0
    assert abs(roof["achieved"] - ops / 0.1 / 1e12) < 1e-6 and roof["launches"] == 9
    assert roof["frac"] == roof["frac_dense"] and abs(roof["frac_own_work"] - 0.6 * roof["frac_dense"]) < 1e-12
    # every operand read once, every output written once: (2560 + 6912) ciphertexts at 16 limbs, (6912 + 2560) at 15
    assert abs(roof["algorithmic_bytes_per_launch"] * 9 - (9472 * 2 * 16 + 9472 * 2 * 15) * 8.0 * 65536) < 1.0
    w = wl.BY_NAME["attn2560"]
    _, roof = bench.roofline_for(w, {"accumulate_mfma": (50.0, 3)})
    assert abs(roof["achieved"] - 2.0 * 2560 * 2560 * 2 * 16 * 65536 * 7 / 0.05 / 1e12) < 1e-6


def test_profile_facts_come_from_the_tracked_summary_or_not_at_all(tmp_path, monkeypatch):
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.profile_facts("ffn2560", "accumulate_mfma") == {}
    (tmp_path / "profiles").mkdir()
    (tmp_path / "profiles" / "bench_ffn2560_kernels_and_hbm_counters.txt").write_text(
        "# text\n@facts accumulate_mfma fetch_GiB_per_step=10.5 write_GiB_per_step=2 mfma_busy=0.6\n@facts other fetch_GiB_per_step=1\n")
    f = bench.profile_facts("ffn2560", "accumulate_mfma")
    assert f == {"fetch_GiB_per_step": 10.5, "write_GiB_per_step": 2.0, "mfma_busy": 0.6}
    _, roof = bench.roofline_for(wl.BY_NAME["ffn2560"], {"accumulate_mfma": (100.0, 5)})
    assert abs(roof["traffic"] - 12.5 * 2 ** 30 / 5) < 1e-3 and roof["mfma_busy"] == 0.6 and roof["valu_util"] is None


def test_plaintext_multiplication_counts():
    w = wl.BY_NAME["merge1536"]  # 1536 products into 96 outputs at 16 limbs
    unit = 8.0 * w.N
    _, roof = bench.roofline_for(w, {"pm_frows_mac_irows": (1.0, 3)})
    assert abs(roof["achieved"] - (1536 + 96) * 2 * 16 * unit / 1e-3 / 1e9) < 1e-6
    w = wl.BY_NAME["rope1536"]  # 96 ciphertexts: 3 products each, 2 rotations sharing one raise
    _, roof = bench.roofline_for(w, {"pm_fcols": (1.0, 3)})
    assert abs(roof["achieved"] - 3 * 96 * 4 * 16 * unit / 1e-3 / 1e9) < 1e-6
    _, roof = bench.roofline_for(w, {"ks_pre": (1.0, 3)})
    assert abs(roof["achieved"] - 96 * 2 * 16 * unit / 1e-3 / 1e9) < 1e-6


def test_giant_and_baby_step_counts():
    w = wl.BY_NAME["ccmmqkbsgs"]  # 96 segments and 1536 elements at period 16, blocks of 2048; 16 + 4 limbs, alpha 4
    assert bench.fill_counts(16, 2048) == (10, 4) and bench.fill_counts(1, 16) == (6, 2)
    unit = 8.0 * w.N
    _, roof = bench.roofline_for(w, {"ks_pre": (1.0, 1)})
    # raises: 96 inputs at 16 limbs; per segment 4 fill groups and one for its baby rotations at 15; per element 2 and per output 1 at 14
    raises = 96 * 2 * 16 + 96 * (4 + 1) * 2 * 15 + (1536 * 2 + 16) * 2 * 14
    assert abs(roof["achieved"] - raises * unit / 1e-3 / 1e9) < 1e-6
    _, roof = bench.roofline_for(w, {"pm_fcols": (1.0, 1)})
    assert abs(roof["achieved"] - (96 * 4 * 16 + 1536 * 4 * 15) * unit / 1e-3 / 1e9) < 1e-6
    w = wl.BY_NAME["ccmmav"]  # one column of V: 32 segments, 512 elements
    _, roof = bench.roofline_for(w, {"ks_icols_special": (1.0, 1)})
    switches = 32 + (32 * 4 + 512) + (512 * 2 + 1)
    assert abs(roof["achieved"] - switches * 4 * 4 * unit / 1e-3 / 1e9) < 1e-6


def test_segment_form_counts():
    w = wl.BY_NAME["ccmmqkseg"]  # 96 ciphertexts of K and of Q, period 64 in baby steps of 4: 127 diagonals, 32 giant steps
    assert (w.period, w.baby, w.d_out) == (64, 4, 64) and bench.fill_counts(64, 2048) == (7, 3)
    unit = 8.0 * w.N
    _, roof = bench.roofline_for(w, {"ks_icols_special": (1.0, 1)})
    # aligning rotations; fill groups and baby steps of K's operands, relinearisations, giant steps of 123 sums (Q's columns are moved outside)
    switches = 96 + (96 * 3 + 96 * 3 + 127 + 123)
    assert abs(roof["achieved"] - switches * 4 * 4 * unit / 1e-3 / 1e9) < 1e-6
    _, roof = bench.roofline_for(w, {"pm_fcols": (1.0, 1)})  # 96 head-mask sources at 16 limbs, the 127 diagonals at 14 (each once)
    assert abs(roof["achieved"] - (96 * 4 * 16 + 127 * 4 * 14) * unit / 1e-3 / 1e9) < 1e-6
    _, roof = bench.roofline_for(w, {"pm_frows_mac_irows": (1.0, 1)})  # 96 + 6112 products read, 96 + 64 sums written
    assert abs(roof["achieved"] - ((96 + 96) * 2 * 16 + (4096 + 2016 + 64) * 2 * 14) * unit / 1e-3 / 1e9) < 1e-6
    # library transforms of the products: 96 * 4 operands (two polynomials of 15 limbs, two passes, in and out), 127 x 3 sums back
    _, roof = bench.roofline_for(w, {"ntt_fwd_cols": (1.0, 1)})
    assert abs(roof["achieved"] - 4 * (96 * 4 * 2 * 15 + 127 * 3 * 15) * unit / 1e-3 / 1e9) < 1e-6
    w = wl.BY_NAME["ccmmavseg"]  # one column of V, 8 segments of 64 tokens, baby steps of 8: 16 giant steps
    assert (w.period, w.baby) == (64, 8)
    _, roof = bench.roofline_for(w, {"ks_pre": (1.0, 1)})
    # raises: the column at 16 limbs; per segment 3 fill groups and one for its baby steps, the 16 relinearisations and the 15 giant steps
    # of the sums, at 15
    assert abs(roof["achieved"] - (1 * 2 * 16 + (8 * 4 + 16 + 15) * 2 * 15) * unit / 1e-3 / 1e9) < 1e-6
