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


def test_issue_report_turns_instruction_counts_into_a_share_of_the_duration(tmp_path):
    k = "void autosage::(anonymous namespace)::softmax_groups_kernel<8, 1, 8>(autosage::(anonymous namespace)::SoftmaxDev)"
    other = "void autosage::spmm_rows_kernel<float, 4, 16, 1, 4, 1, false>(autosage::SpmmDev)"
    dur = 1_000_000                                         # 1 ms = 2.4e6 cycles
    valu = 0.5 * 2.4e6 * 1024 / 4                           # issuing these takes half of the duration on 1024 SIMDs
    rows = []
    for i in range(3):
        rows += [(k, "SQ_WAVES", 1000.0, i, dur), (k, "SQ_INSTS_VALU", valu, i, dur), (k, "SQ_INSTS_SALU", 50_000.0, i, dur),
                 (k, "SQ_INSTS_LDS", 10_000.0, i, dur), (k, "SQ_INSTS_VMEM_RD", 8_000.0, i, dur)]
    rows += [(other, "SQ_WAVES", 10.0, 9, dur), (other, "SQ_INSTS_VALU", 100.0, 9, dur)]
    p = str(tmp_path / "sq.db")
    make_db(p, [], rows)
    lines = [l for l in R.issue_report(p, last=3, match="softmax").split("\n") if l.startswith("| `")]
    assert len(lines) == 1 and "softmax_groups_kernel<8, 1, 8>" in lines[0]
    c = [x.strip() for x in lines[0].strip("|").split("|")]
    assert c[1] == "3" and float(c[2]) == 1.0 and float(c[3]) == 1000 and float(c[4]) == round(valu / 1000)
    assert c[5] == "50" and c[6] == "10" and c[7] == "8.0" and c[8] == "50 %"
