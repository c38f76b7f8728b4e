"""Host-side pieces of the benchmark: the counter summary (rocprofv3 CSV -> markdown) and the way bench.py quotes it."""
import csv
import io
import os
import sys
from contextlib import redirect_stdout

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _write_counter_csv(path, counter, rows):
    """rows: (kernel name, grid, KiB).  Dispatch ids follow the list order."""
    cols = ["Correlation_Id", "Dispatch_Id", "Agent_Id", "Queue_Id", "Process_Id", "Thread_Id", "Grid_Size", "Kernel_Id",
            "Kernel_Name", "Workgroup_Size", "LDS_Block_Size", "Scratch_Size", "VGPR_Count", "Accum_VGPR_Count", "SGPR_Count",
            "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"]
    with open(path, "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=cols)
        w.writeheader()
        for i, (name, grid, kib) in enumerate(rows, start=1):
            r = dict.fromkeys(cols, 0)
            r.update(Dispatch_Id=i, Grid_Size=grid, Kernel_Name=name, Counter_Name=counter, Counter_Value=kib)
            w.writerow(r)


def _run(scale):
    """One synthetic run: a plain call, a prepared call and a folded call (each a recode launch then the GEMM),
    a whole-word ReLU call with the copy exchange and one with the remote store."""
    A = "(anonymous namespace)::"
    gemm = f"void {A}k_limb_gemm<2, 2, true>(GemmArgs)"
    rec = f"{A}k_recode_mixed({A}RecodeMixed)"
    rows = f"{A}k_recode_rows({A}RecodeArgs)"
    st = lambda s, put: f"void {A}k_relu_stage<{s}, 4, 0, {'true' if put else 'false'}>({A}ReluParty, {A}ReluParty, int, unsigned long, unsigned long)"
    wire = f"void {A}k_wire_words<4>(unsigned long const*, unsigned long*)"
    out = [("void at::native::something<int>(int)", 512, 999.0),                    # torch: ignored
            (f"void {A}k_sub_multi<false>(SubBatch)", 4194304, 70144.0 * scale),
            (f"{A}k_copy_multi(CopyBatch)", 4194304, 35072.0 * scale),               # the calibration kernel
            (rec, 422400, 100.0), (gemm, 131072, 135.0 * 1024 * scale),              # plain call
            (rec, 131584, 100.0), (gemm, 131072, 135.0 * 1024 * scale),              # prepared call
            (rec, 263168, 100.0), (gemm, 131072, 110.0 * 1024 * scale),              # folded call, copy exchange
            (rows, 65792, 50.0), (rows, 65792, 50.0), (gemm, 131072, 108.0 * 1024 * scale),      # folded call, remote store
            (gemm, 65536, 25.0 * 1024 * scale)]                                      # a dealer launch (smaller grid)
    relu_copy = [(wire, 1048576, 1000.0 * scale)] + [(st(s, False), 524288, 2000.0 * scale) for s in range(10)]
    relu_put = [(st(s, s < 9), 524288, 1500.0 * scale) for s in range(10)]
    # two chunks per call, calls separated by a conv-call kernel
    out += relu_copy + relu_copy + [(rec, 263168, 100.0)] + relu_put + relu_put + [(rec, 263168, 100.0)]
    return out


def test_pmc_summary_and_bench_quote(tmp_path, monkeypatch):
    import bench
    from paper_2209_13643_amd import pmc_summary
    f, w = tmp_path / "f.csv", tmp_path / "w.csv"
    _write_counter_csv(f, "FETCH_SIZE", _run(0.5))        # the fetch counter reads half the bytes: scale x2
    _write_counter_csv(w, "WRITE_SIZE", _run(1.0))
    out = io.StringIO()
    with redirect_stdout(out):
        assert pmc_summary.main([str(f), str(w)]) == 0
    text = out.getvalue()
    assert "scale x2.000" in text and "scale x1.000" in text
    assert f"sources sha256/16: {pmc_summary.sources_digest()}" in text
    assert "| k_limb_gemm in the folded prepared call (three products) | 108.0 | 108.0 |" in text
    assert "| k_limb_gemm in the plain call (four products) | 135.0 | 135.0 |" in text
    assert "| k_limb_gemm in the folded prepared call with the copy exchange (three products) | 110.0 | 110.0 |" in text
    n = 64 * 16 * 16 * 128
    per_call_copy = 2 * (1000.0 + 10 * 2000.0) * 1024 * 2            # two chunks, fetch + write after scaling
    assert f"whole words, exchange by copy, all kernels of one call (both parties + wire), {n} elements" in text
    assert f"= {per_call_copy / n:.0f} bytes per element" in text
    per_call_put = 2 * (10 * 1500.0) * 1024 * 2
    assert f"= {per_call_put / n:.0f} bytes per element" in text
    # bench.py quotes the summary while the digest matches the sources ...
    md = tmp_path / "summary.md"
    md.write_text(text)
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    monkeypatch.setattr(bench, "sources_digest", pmc_summary.sources_digest)
    q = bench.read_pmc_summary(str(md))
    assert q is not None and q["measured_in_this_run"] is False
    assert q["fetch_bytes"] == 108.0 * 2 ** 20 and q["write_bytes"] == 108.0 * 2 ** 20      # the folded call's launch
    assert q["four_product_launch"]["fetch_bytes"] == 135.0 * 2 ** 20
    assert q["relu_bytes_per_element"] == round(per_call_copy / n)
    assert q["relu_put_bytes_per_element"] == round(per_call_put / n)
    # ... and not once they differ, or when there is no such file
    md.write_text(text.replace(pmc_summary.sources_digest(), "0" * 16))
    assert bench.read_pmc_summary(str(md)) is None
    assert bench.read_pmc_summary(str(tmp_path / "missing.md")) is None


def test_digests_agree():
    import bench
    from paper_2209_13643_amd import pmc_summary
    assert bench.sources_digest() == pmc_summary.sources_digest()
