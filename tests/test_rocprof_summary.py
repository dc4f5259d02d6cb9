"""Host logic of the profile summariser: counter scaling by the copy probe and the text round trip."""
import csv

from paper_2502_02581_amd import rocprof_summary as rs

FIELDS = ["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"]


def write_csv(path, rows):
    with open(path, "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=FIELDS)
        w.writeheader()
        for r in rows:
            w.writerow(dict(zip(FIELDS, r)))


def test_traffic_scaled_by_copy_probe(tmp_path):
    probe = "void moe::copy_probe_kernel(unsigned int const*, unsigned int*, unsigned long)"
    kern = "void moe::row_gemm_kernel<moe::RowCores<2, 2, false>, 2, 1, false>(moe::RowGemm)"
    fetch, write = tmp_path / "f.csv", tmp_path / "w.csv"
    # the probe moves 1000 bytes each way; FETCH_SIZE prices them as 50 units, WRITE_SIZE as 100
    write_csv(fetch, [(1, probe, "FETCH_SIZE", 50), (2, kern, "FETCH_SIZE", 300), (3, kern, "FETCH_SIZE", 100),
                      (4, "void at::native::copy()", "FETCH_SIZE", 7)])
    write_csv(write, [(1, probe, "WRITE_SIZE", 100), (2, kern, "WRITE_SIZE", 10), (3, kern, "WRITE_SIZE", 30)])
    out = tmp_path / "t.txt"

    class A:
        fetch_csv, write_csv, probe_bytes, cmd, commit = str(fetch), str(write), 1000, "cmd", "abc1234"

    A.out = str(out)
    rs.traffic(A)
    got = rs.read_traffic(str(out))
    name = kern.replace("void moe::", "moe::")
    # per launch: fetched (300 + 100) / 2 * 20 B = 4000, written (10 + 30) / 2 * 10 B = 200
    assert got[name] == 4200.0
    assert got[probe.replace("void moe::", "moe::")] == 2000.0
    assert not any("at::native" in k for k in got)
    assert "# commit: abc1234" in out.read_text()


def test_counters_ratios(tmp_path):
    kern = "void moe::w_gemm_kernel<moe::MfmaDmaCore<256, 256, 1, false, false, 2, 4, 1>, 1>(moe::WGemm)"
    c = tmp_path / "c.csv"
    write_csv(c, [(1, kern, "SQ_VALU_MFMA_BUSY_CYCLES", 200), (1, kern, "SQ_BUSY_CU_CYCLES", 100),
                  (1, kern, "SQ_INSTS_VALU_MFMA_MOPS_BF16", 2e9), (1, kern, "SQ_LDS_BANK_CONFLICT", 5),
                  (1, kern, "SQ_LDS_IDX_ACTIVE", 50)])
    out = tmp_path / "c.md"

    class A:
        csv, cmd, commit = [str(c)], ["cmd one"], "abc1234"

    A.out = str(out)
    rs.counters(A)
    text = out.read_text()
    assert "MFMA busy                          0.500" in text
    assert "executed bf16 MFMA TFLOP           1.024" in text
    assert "LDS bank conflict share            0.100" in text
