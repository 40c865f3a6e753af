"""bench.py's bookkeeping, without a GPU: the source fingerprint that ties a rocprofv3 summary under profiles/
to the build it was taken with, and the reading of the counter bytes from such a summary."""
import os
import shutil

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_fingerprint_ignores_comments_and_layout_but_not_code(tmp_path, monkeypatch):
    src = tmp_path / "csrc"
    shutil.copytree(bench.CSRC, src)
    monkeypatch.setattr(bench, "CSRC", str(src))
    base = bench.library_fingerprint()
    f = src / "device_utils.h"
    text = f.read_text()
    f.write_text("// a remark\n" + text.replace("constexpr int kWave = 64;", "constexpr int kWave   =   64;   /* lanes */"))
    assert bench.library_fingerprint() == base
    f.write_text(text.replace("constexpr int kWave = 64;", "constexpr int kWave = 32;"))
    assert bench.library_fingerprint() != base


def test_counter_bytes_come_from_the_matching_summary_or_are_null(tmp_path, monkeypatch):
    w = "cfg4_topk_n8_d110000000"
    got, source = bench.measured_traffic(w, "ef", "tk_pass1")
    if got is not None:                       # the committed summary matches the tree
        assert source == f"profiles/{w}.md" and 10.5e9 < got < 10.8e9      # 12 n d = 10.56 GB plus the candidates
    else:
        assert "was taken with sources" in source
    # a summary taken with other sources is refused, and the reason names both fingerprints
    monkeypatch.setattr(bench, "library_fingerprint", lambda: "000000000000")
    got, source = bench.measured_traffic(w, "ef", "tk_pass1")
    assert got is None and "000000000000" in source
    # no summary for the workload, or none for the combination of method and gradient type
    assert bench.measured_traffic("no_such_workload", "ef", "tk_pass1")[0] is None
    assert bench.measured_traffic(w, None, "tk_pass1")[0] is None


def test_which_summary_a_run_reads():
    assert bench.run_variant("ef", "f32", False) == "ef"
    assert bench.run_variant("cd", "f32", False) == "cd"
    assert bench.run_variant("naive", "f32", False) == "naive"
    assert bench.run_variant("ef", "bf16", False) == "bf16"
    assert bench.run_variant("ef", "f32", True) == "randk"
    assert bench.run_variant("cd", "bf16", False) is None
    assert bench.run_variant("ef", "f16", False) is None
    assert bench.run_variant("cd", "f32", True) is None
    assert set(bench.PROFILE_SUFFIX) == {"ef", "cd", "naive", "none", "bf16", "randk"}
