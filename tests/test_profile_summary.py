"""The profile summariser turns rocprofv3 CSV files into the figures quoted for the kernels (clock,
matrix-pipe and LDS occupancy, HBM traffic).  Here it runs on small hand-made CSV files whose
answers are known, so that the arithmetic behind those figures is pinned."""
import csv
import json
import os

from paper_2503_12964_amd import profile_summary as PS

DKDV = "void vfm::attn_bwd_dkdv_kernel<128, vfm::SegTable, false>(...)"
DQ2 = "_ZN3vfm19attn_bwd_dq2_kernelILi128ENS_8SegTableEEEvPKDF16b"
FWD = "_ZN3vfm15attn_fwd_kernelILi128ELi8ENS_8SegTableEEEvPKDF16b"
PREP = "void vfm::bwd_prepare_kernel<128>(...)"
COPY = "__amd_rocclr_copyBuffer"


def _stats(path, rows):
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"])
        for name, calls, avg_ns, pct in rows:
            w.writerow([name, calls, calls * avg_ns, avg_ns, pct, avg_ns - 1, avg_ns + 1, 0.0])


def _pmc(path, rows):
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"])
        for i, (name, counter, value) in enumerate(rows):
            w.writerow([i, name, counter, value])


def _bench_line(path, fwd_ms, bwd_ms):
    line = {"metric": "m", "value": 1000.0, "unit": "TFLOP/s", "steps": 5, "warmup": 2, "ms_per_step": fwd_ms + bwd_ms,
            "config": {"workload": "C4: test"},
            "breakdown": {"fwd_ms": fwd_ms, "bwd_ms": bwd_ms, "rope_ms": 0.3},
            "roofline": {"achieved": 900.0, "frac": 0.36, "kernel": "k", "bound": "mfma", "unit": "TFLOP/s"}}
    open(path, "w").write("noise\n" + json.dumps(line) + "\n")


def test_headline_summary_arithmetic(tmp_path, monkeypatch):
    run = tmp_path / "run"
    run.mkdir()
    monkeypatch.setattr(PS, "TRAFFIC_FILE", str(tmp_path / "traffic.txt"))
    # kernel times: 80 ms, 50 ms, 40 ms, 0.2 ms
    _stats(run / "stats_kernel_stats.csv", [(DKDV, 7, 80e6, 46.0), (DQ2, 7, 50e6, 29.0), (FWD, 7, 40e6, 23.0),
                                           (PREP, 7, 0.2e6, 0.1)])
    _bench_line(run / "stats.log", 40.0, 130.2)
    # a 1 GiB copy for which FETCH_SIZE reads half and WRITE_SIZE all of it -> scale factors 2 and 1
    _pmc(run / "cal_fetch_counter_collection.csv", [(COPY, "FETCH_SIZE", 524288.0)])
    _pmc(run / "cal_write_counter_collection.csv", [(COPY, "WRITE_SIZE", 1048576.0)])
    # two dispatches per kernel: the mean counts
    _pmc(run / "fetch_counter_collection.csv", [(DKDV, "FETCH_SIZE", 6e6), (DKDV, "FETCH_SIZE", 8e6),
                                                (DQ2, "FETCH_SIZE", 4e6), (FWD, "FETCH_SIZE", 3e6),
                                                (PREP, "FETCH_SIZE", 0.5e6)])
    _pmc(run / "write_counter_collection.csv", [(DKDV, "WRITE_SIZE", 1e6), (DQ2, "WRITE_SIZE", 0.5e6),
                                                (FWD, "WRITE_SIZE", 0.5e6), (PREP, "WRITE_SIZE", 0.0)])
    # dK/dV kernel: clocked 1.6 GHz for 80 ms on each of the 32 shader engines; the matrix pipe busy 3/4 of it
    cyc = 1.6e9 * 80e-3
    _pmc(run / "sq_counter_collection.csv", [(DKDV, "SQ_BUSY_CYCLES", cyc * PS.N_SE),
                                             (DKDV, "SQ_VALU_MFMA_BUSY_CYCLES", 0.75 * cyc * PS.N_SIMD),
                                             (DKDV, "SQ_INSTS_MFMA", 3e9), (DKDV, "SQ_INSTS_VALU", 1e10),
                                             (DKDV, "SQ_LDS_BANK_CONFLICT", 0.0)])
    _pmc(run / "lds_counter_collection.csv", [(DKDV, "SQ_BUSY_CYCLES", cyc * PS.N_SE),
                                              (DKDV, "SQ_LDS_IDX_ACTIVE", 0.5 * cyc * PS.N_CU),
                                              (DKDV, "SQ_WAVE_CYCLES", 1e10), (DKDV, "SQ_WAIT_INST_LDS", 1e9),
                                              (DKDV, "SQ_ACTIVE_INST_VALU", 4e9), (DKDV, "SQ_INSTS_LDS", 5e9),
                                              (DKDV, "SQ_INSTS_VALU_TRANS_F32", 1.5e9)])
    text = PS.summarise(str(run), "C4", str(tmp_path / "out.txt"))
    assert (tmp_path / "out.txt").read_text() == text

    def row(section_marker, label):
        sec = text[text.index(section_marker):]
        return next(l for l in sec.splitlines() if l.strip().startswith(label)).split()

    # [1] kernel times and their sum against the bench line's backward time
    assert row("[1]", "attn_bwd_dkdv_kernel")[2] == "80.000"
    assert "backward kernels summed: 130.200 ms" in text and "130.200 ms)" in text
    # [2] scale factors and scaled traffic: dK/dV mean fetch 7e6 KiB x 2 x 1024 B = 14.336 GB, writes 1.024 GB
    assert "scale 2.0000" in text and "scale 1.0000" in text
    r = row("[2]", "attn_bwd_dkdv_kernel")
    assert r[1:] == ["7000000", "1000000", "14.336", "1.024"]
    bwd = (7e6 * 2 + 1e6 + 4e6 * 2 + 0.5e6 + 0.5e6 * 2) * 1024
    fwd = (3e6 * 2 + 0.5e6) * 1024
    traffic = dict(l.split()[1:] for l in open(tmp_path / "traffic.txt") if l.startswith("C4"))
    assert abs(float(traffic["backward_call"]) - bwd) < 1e-6 * bwd and abs(float(traffic["forward_call"]) - fwd) < 1e-6 * fwd
    # [3] clock from SQ_BUSY_CYCLES, occupancy at the nominal and at the measured clock
    r = row("[3]", "attn_bwd_dkdv_kernel")
    assert r[3] == "1.60" and r[4] == "0.500" and r[5] == "0.750"       # 0.75 * 1.6 / 2.4 = 0.5
    # [4] LDS pipe busy, waits and VALU activity as shares
    r = row("[4]", "attn_bwd_dkdv_kernel")
    assert r[3] == "0.500" and r[4] == "0.100" and r[6] == "0.400"


def test_traffic_file_keeps_other_workloads(tmp_path, monkeypatch):
    path = tmp_path / "traffic.txt"
    monkeypatch.setattr(PS, "TRAFFIC_FILE", str(path))
    PS._write_traffic("C4", {"backward_call": 2.5e10, "forward_call": 8e9})
    PS._write_traffic("P256", {"backward_call": 6e9, "forward_call": 2e9})
    PS._write_traffic("C4", {"backward_call": 2.4e10, "forward_call": 8.1e9})
    lines = [l.split() for l in open(path) if not l.startswith("#")]
    assert sorted(l[0] for l in lines) == ["C4", "C4", "P256", "P256"]
    assert ["C4", "backward_call", "2.400000e+10"] in lines and ["P256", "forward_call", "2.000000e+09"] in lines


def test_kernel_labels():
    assert PS._label("void vfm::tattn_fwd_kernel<128>(...)") == "tattn_fwd_kernel"
    assert PS._label("_ZN3vfm20attn_bwd_both_kernelILi128E") == "attn_bwd_both_kernel"
    assert PS._label("_ZN3vfm19attn_fwd_fp8_kernelILi128E") == "attn_fwd_fp8_kernel"
    assert PS._label("void vfm::qknorm_rope3d_bwd_kernel<128>(...)").startswith("qknorm_rope3d_bwd_kernel")
    assert PS._label("some_other_kernel") is None
    assert PS._short_kernel("_ZN3vfm17tattnL_fwd_kernelILi128ELb1EEEvPKDF16b") == "tattnL_fwd_kernel (bwd stats)"
    assert PS._short_kernel("void vfm::tattnL_fwd_kernel<128, false>(...)") == "tattnL_fwd_kernel (forward)"
