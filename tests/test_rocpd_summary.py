"""The profile summariser on a hand-made database with the two views it reads (CPU only)."""
import sqlite3

from paper_2511_17594_amd import rocpd_summary as R


def make_db(path, kernels, counters):
    db = sqlite3.connect(path)
    db.execute("create table kernels (name text, start integer, duration integer)")
    db.execute("create table counters_collection (kernel_name text, counter_name text, value real, start integer, duration integer)")
    db.executemany("insert into kernels values (?, ?, ?)", kernels)
    db.executemany("insert into counters_collection values (?, ?, ?, ?, ?)", counters)
    db.commit()
    db.close()


def test_kernel_table_separates_probe_dispatches_from_timed_steps(tmp_path):
    name = "void autosage::spmm_rows_kernel<float, 4, 16, 1, 4, 1, false>(autosage::SpmmDev)"
    rows = [(name, i, 100_000) for i in range(4)] + [(name, 10 + i, 1_000_000) for i in range(3)]
    rows.append(("autosage::(anonymous namespace)::hub_fill_kernel(autosage::PartDev)", 50, 5_000))
    p = str(tmp_path / "kt.db")
    make_db(p, rows, [])
    lines = R.kernel_table(p, last=3).split("\n")
    spmm = [l for l in lines if "spmm_rows_kernel<float, 4, 16, 1, 4, 1, false>" in l][0].split("|")
    assert "autosage::" not in spmm[1] and "(" not in spmm[1]
    assert int(spmm[2]) == 7
    assert abs(float(spmm[4]) - 3.4 / 7) < 1e-3            # all dispatches
    assert abs(float(spmm[5]) - 1.0) < 1e-9                # the last three only


def test_counter_report_scales_by_the_copy_calibration(tmp_path):
    gib = 1 << 30
    copy = "__amd_rocclr_copyBuffer"
    k = "void autosage::attn_fused_rows_kernel<autosage::bf16_t, 8, 8, 8, 1, 4>(autosage::AttnDev)"
    fetch = [(copy, "FETCH_SIZE", gib / 2048, i, 400_000) for i in range(3)]
    fetch += [(k, "FETCH_SIZE", 1000.0, 10, 50_000)] + [(k, "FETCH_SIZE", 4_000_000.0, 20 + i, 1_300_000) for i in range(5)]
    write = [(copy, "WRITE_SIZE", gib / 1024, i, 400_000) for i in range(3)]
    write += [(k, "WRITE_SIZE", 10.0, 10, 50_000)] + [(k, "WRITE_SIZE", 500_000.0, 20 + i, 1_300_000) for i in range(5)]
    pf, pw = str(tmp_path / "f.db"), str(tmp_path / "w.db")
    make_db(pf, [], fetch)
    make_db(pw, [], write)
    assert abs(R.bytes_per_unit(R.counter_samples(pf)) - 2048.0) < 1e-9
    text, traffic = R.counter_report(pf, pw, last=5)
    assert traffic == ["attn_fused_rows %d" % (4_000_000 * 2048 + 500_000 * 1024)]
    assert "attn_fused_rows" in text and "copyBuffer" not in text.split("|---")[1]
    out = R.fetch_report(pf, last=5)
    assert "8192.0" in out                                   # MB read per launch
