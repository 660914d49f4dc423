"""Host-side pieces around the measurements: bench.py's refusal of more than one GPU, and the summaries of rocprofv3
output that link a profile to the kernel sources it was measured on (paper_2202_12429_amd/profile_summary.py)."""
import os
import subprocess
import sys

from paper_2202_12429_amd import profile_summary as ps

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0
    assert "single-GPU" in r.stderr + r.stdout


def test_kernel_source_digest_follows_the_sources(tmp_path, monkeypatch):
    a = ps.kernel_source_digest()
    assert len(a) == 16 and a == ps.kernel_source_digest()
    # another csrc directory with one more byte gives another digest
    csrc = tmp_path / "pkg" / "csrc"
    csrc.mkdir(parents=True)
    (tmp_path / "include").mkdir()
    (tmp_path / "include" / "bagpipe.h").write_text("header")
    (csrc / "k.hip").write_text("kernel")
    monkeypatch.setattr(ps, "HERE", str(tmp_path / "pkg"))
    monkeypatch.setattr(ps, "ROOT", str(tmp_path))
    b = ps.kernel_source_digest()
    (csrc / "k.hip").write_text("kernel ")
    c = ps.kernel_source_digest()
    assert len({a, b, c}) == 3


def test_short_kernel_name():
    full = "void bp::(anonymous namespace)::bwd_rows_kernel<16, false>(HIP_vector_type<unsigned int, 4u> const*, ...)"
    assert ps.short_kernel_name(full) == "bwd_rows_kernel<16, false>"
    assert ps.short_kernel_name("void bp::sort_upsweep_kernel<unsigned long, 16, 9, bp::SortArrays<unsigned long> >(...)") == \
        "sort_upsweep_kernel<u64, 16, 9, SortArrays<u64> >"
    assert ps.short_kernel_name("at::native::vectorized_elementwise_kernel<4, ...>") == ""


def write_csv(path, header, rows):
    path.parent.mkdir(parents=True, exist_ok=True)
    path.write_text(",".join(header) + "\n" + "".join(",".join(f'"{c}"' for c in r) + "\n" for r in rows))


def test_stats_and_pmc_summaries(tmp_path):
    k = "void bp::(anonymous namespace)::bwd_rows_kernel<16, false>(int)"
    c = "void bp::copy_calibration_kernel(float*)"
    write_csv(tmp_path / "x" / "run_kernel_trace.csv", ["Kernel_Name", "Start_Timestamp", "End_Timestamp"],
              [[k, 1000, 41000], [k, 50000, 88000], ["other_kernel", 0, 5], [c, 100000, 450000]])
    text = ps.stats_summary(str(tmp_path), "run")
    lines = text.splitlines()
    assert lines[0].startswith(ps.DIGEST_TAG)
    row = next(l for l in lines if l.startswith("bwd_rows_kernel<16, false>")).split()
    assert row[-6:] == ["2", "39.00", "39.00", "38.00", "40.00", "0.078"]
    assert not any("other_kernel" in l for l in lines)

    kib = 2 ** 30 / 1024
    hdr = ["Kernel_Name", "Counter_Value"]
    write_csv(tmp_path / "p" / "pmc_FETCH_SIZE_counter_collection.csv", hdr, [[c, kib / 2], [k, 50000], [k, 70000]])
    write_csv(tmp_path / "p" / "pmc_WRITE_SIZE_counter_collection.csv", hdr, [[c, kib], [k, 30000], [k, 30000]])
    out = tmp_path / "pmc.txt"
    out.write_text("some header\n" + ps.pmc_summary(str(tmp_path / "p")) + "\n")
    digest, traffic = ps.read_traffic(str(out))
    assert digest == ps.kernel_source_digest()
    # fetch counts half the bytes (x2), write all of them: (2 * 60000 + 30000) KiB
    assert traffic["bwd_rows_kernel"] == (2 * 60000 + 30000) * 1024
    assert ps.read_traffic(str(tmp_path / "absent.txt")) == (None, {})
