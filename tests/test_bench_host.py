"""Host logic of bench.py (no GPU): the refusal of more than one GPU, the algorithmic bytes and flops that the
roofline figures divide by, the guard on the recorded HBM traffic, and the kernel-trace summary."""
import os
import subprocess
import sys
import types

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_work_is_the_per_unit_figures_summed_over_the_batch():
    """Per decode row c*2*Hkv*D*s_kv + 2*Hq*D*s_q + ceil(c/16)*4 bytes and 4*Hq*D*c flop; per chunk
    4*Hq*D*(q*p + q(q+1)/2) flop and (p+q)*2*Hkv*D*s_kv + 2*q*Hq*D*s_q bytes; 2*Hkv*D*(s_q+s_kv) append bytes per
    new token -- written out by hand for two rows and a chunk."""
    shape = types.SimpleNamespace(num_q_heads=8, num_kv_heads=2, head_dim=128, q_dtype="bf16", kv_dtype="fp8")
    batch = types.SimpleNamespace(shape=shape, q_lens=np.array([1, 1, 10, 0], np.int32), ctx_lens=np.array([17, 100, 30, 5], np.int32))
    w = bench.algorithmic_work(batch)
    assert w["decode_bytes"] == (17 * 2 * 2 * 128 * 1 + 2 * 8 * 128 * 2 + 2 * 4) + (100 * 2 * 2 * 128 * 1 + 2 * 8 * 128 * 2 + 7 * 4)
    assert w["decode_flops"] == 4 * 8 * 128 * (17 + 100)
    assert w["prefill_flops"] == 4 * 8 * 128 * (10 * 20 + 55)
    assert w["prefill_bytes"] == 30 * 2 * 2 * 128 * 1 + 2 * 10 * 8 * 128 * 2
    assert w["append_bytes"] == 12 * 2 * 2 * 128 * (2 + 1)


def test_recorded_traffic_is_dropped_when_the_kernel_sources_change(tmp_path, monkeypatch):
    import hashlib
    csrc = tmp_path / "paper_2512_03416_amd" / "csrc"
    csrc.mkdir(parents=True)
    (tmp_path / "profiles").mkdir()
    (csrc / "a.h").write_text("kernel one")
    (csrc / "b.hip").write_text("kernel two")
    digest = hashlib.sha256(b"kernel one" + b"kernel two").hexdigest()
    (tmp_path / "profiles" / "some_kernel_cfg9_traffic.txt").write_text(
        f"# comment\nworkload=cfg9_thing\nfetch_bytes=1000\nwrite_bytes=24\nsources=a.h,b.hip\ndigest={digest}\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.recorded_traffic("some_kernel", "cfg9_thing") == 1024
    assert bench.recorded_traffic("some_kernel", "cfg9_other") is None          # another workload's figure
    assert bench.recorded_traffic("other_kernel", "cfg9_thing") is None         # no file
    (csrc / "b.hip").write_text("kernel two, changed")
    assert bench.recorded_traffic("some_kernel", "cfg9_thing") is None


def test_the_committed_traffic_figures_parse():
    """Every traffic file under profiles/ names its workload, both byte counts, its sources (which exist) and a digest."""
    import glob
    files = glob.glob(os.path.join(ROOT, "profiles", "*_traffic.txt"))
    assert files
    for f in files:
        kv = dict(l.strip().split("=", 1) for l in open(f) if "=" in l and not l.startswith("#"))
        assert int(kv["fetch_bytes"]) > 0 and int(kv["write_bytes"]) > 0 and len(kv["digest"]) == 64 and kv["workload"]
        for s in kv["sources"].split(","):
            assert os.path.exists(os.path.join(ROOT, "paper_2512_03416_amd", "csrc", s)), s


def test_trace_summary_pairs_the_co_resident_kernels(tmp_path, capsys):
    d = tmp_path / "kt" / "host" / "1"
    d.mkdir(parents=True)
    rows = ["Kind,Agent_Id,Queue_Id,Kernel_Name,Start_Timestamp,End_Timestamp"]
    t = 0
    for i in range(3):
        rows.append(f"K,1,1,void ts::append_token_kernel<unsigned short>(ts::AppendArgs),{t},{t + 5000}")
        rows.append(f"K,1,1,\"void ts::prefill_resident_kernel<unsigned short, false>(ts::AttnArgs)\",{t + 10000},{t + 510000}")
        rows.append(f"K,1,2,\"void ts::decode_kernel_lean<unsigned short, 128>(ts::AttnArgs)\",{t + 16000},{t + 610000}")
        rows.append(f"K,1,2,ts::combine_kernel(ts::AttnArgs),{t + 610000},{t + 614000}")
        t += 700000
    (d / "kt_kernel_trace.csv").write_text("\n".join(rows) + "\n")
    bench.summarise_trace(str(tmp_path / "kt"))
    out = capsys.readouterr().out
    assert "| `void ts::prefill_resident_kernel<unsigned short, false>` | 3 | 500.0 | 500.0 | 500.0 |" in out
    assert "co-resident pairs" in out and "(3): span mean 600.0 us" in out
    assert "the decode kernel next to it 594.0 us, started 6.0 us after it" in out
