"""The counter summariser on a synthetic rocpd-like database: scaling by the copy kernel of known size."""
import sqlite3
import subprocess
import sys


def _db(path, rows):
    con = sqlite3.connect(path)
    con.execute("create table counters_collection (kernel_name text, value real)")
    con.executemany("insert into counters_collection values (?, ?)", rows)
    con.commit()
    con.close()


def test_bytes_are_scaled_by_the_copy_kernel(tmp_path):
    copy = "k_probe_copy(HIP_vector_type<unsigned int, 4u> const*, HIP_vector_type<unsigned int, 4u>*, unsigned long)"
    gemv = "void rs::k_gemv<2, 4, 1, 4, 1, 3>(rs::GemvArgs)"
    # the fetch counter under-reads by 2x (as on MI355X), the write counter is exact
    _db(tmp_path / "f.db", [(copy, 131072.0)] * 3 + [(gemv, 65536.0), (gemv, 65536.0), ("other", 5.0)])
    _db(tmp_path / "w.db", [(copy, 262144.0)] * 3 + [(gemv, 1024.0), (gemv, 1024.0)])
    r = subprocess.run([sys.executable, "-m", "paper_2507_17307_amd.pmc_summary", str(tmp_path / "f.db"), str(tmp_path / "w.db")],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    line = [l for l in r.stdout.splitlines() if "k_gemv" in l][0].split()
    # 65536 units x 2048 bytes = 134.218 MB fetched; 1024 units x 1024 bytes = 1.049 MB written
    assert line[-3:] == ["2", "134.218", "1.049"]
    assert "other" not in r.stdout


def test_missing_copy_kernel_is_an_error(tmp_path):
    _db(tmp_path / "f.db", [("void rs::k_gemv<0>(rs::GemvArgs)", 1.0)])
    _db(tmp_path / "w.db", [("void rs::k_gemv<0>(rs::GemvArgs)", 1.0)])
    r = subprocess.run([sys.executable, "-m", "paper_2507_17307_amd.pmc_summary", str(tmp_path / "f.db"), str(tmp_path / "w.db")],
                       capture_output=True, text=True)
    assert r.returncode == 1 and "copy kernel" in r.stderr
