"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode == 2
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_world_size_above_one_is_refused():
    env = dict(os.environ, WORLD_SIZE="2")
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, env=env)
    assert p.returncode == 2


def test_help_lists_the_workloads_and_options():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True)
    assert p.returncode == 0
    for word in ("--steps", "--warmup", "--workload", "--ell", "--adapters", "c5_model", "c4_sweep"):
        assert word in p.stdout


def test_traffic_figure_is_tied_to_the_kernel_sources(tmp_path):
    """bench.py's `traffic` comes from profiles/hbm_traffic.json and is only reported while the hash of the kernel sources
    stored with it matches the sources in the tree; no byte count is typed into bench.py."""
    import json
    from paper_2605_24058_amd import traffic_profile as tp
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert "* 1024}" not in src and "MEASURED_TRAFFIC" not in src
    wl = "c2_llama7b_attn_4096x4096_r16_T2048"
    good = {"entries": [{"call": "lordba_forward", "workload": wl, "variant": "", "bytes_per_call": 123,
                         "source_sha256": tp.source_hash("lordba_forward"), "measured_after_commit": "abc"}]}
    p = tmp_path / "t.json"
    p.write_text(json.dumps(good))
    assert tp.lookup("lordba_forward", wl, path=str(p))[0] == 123
    assert tp.lookup("lordba_forward", "other", path=str(p))[0] is None
    good["entries"][0]["source_sha256"] = "0" * 64
    p.write_text(json.dumps(good))
    val, note = tp.lookup("lordba_forward", wl, path=str(p))
    assert val is None and "changed" in note
    assert tp.lookup("lordba_forward", wl, path=str(tmp_path / "missing.json"))[0] is None
    # the committed file parses, and an entry that matches the tree's sources is what bench.py would report
    doc = json.load(open(tp.DEFAULT_JSON))
    for e in doc["entries"]:
        assert e["bytes_per_call"] > 0 and len(e["source_sha256"]) == 64 and e["kernels"]


def test_counter_csv_parser(tmp_path):
    from paper_2605_24058_amd import traffic_profile as tp
    head = '"Correlation_Id","Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"\n'
    rows = ['1,1,"void (anonymous namespace)::k_a<1, 2>(Args)","FETCH_SIZE",10.0', '2,2,"void (anonymous namespace)::k_b(Args)","FETCH_SIZE",4.0',
            '3,3,"void (anonymous namespace)::k_a<1, 2>(Args)","FETCH_SIZE",14.0', '4,4,"other","FETCH_SIZE",99.0',
            '5,5,"void (anonymous namespace)::k_a<1, 2>(Args)","WRITE_SIZE",1.0']
    p = tmp_path / "c.csv"
    p.write_text(head + "\n".join(rows) + "\n")
    total, detail = tp.kib_per_call(str(p), "FETCH_SIZE", "k_")
    assert total == 28.0 and detail["k_a<1, 2>(Args)"] == (2.0, 12.0) and detail["k_b(Args)"] == (1.0, 4.0)
