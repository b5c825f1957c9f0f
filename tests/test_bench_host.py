"""Host-side checks of the benchmark driver that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300, cwd=ROOT)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus 2" in r.stderr
    assert r.stdout.strip() == ""      # no JSON line for a run that did not happen


def test_byte_and_flop_models_of_the_kernels():
    # The roofline's numerators, re-derived by hand for C = 64, d = 128, bf16.
    sys.path.insert(0, ROOT)
    import bench
    # operand model: per (chunk, head) the chunk kernel reads dO, Ut, dUt, K, Q, V (six 64x128 tiles), S and dS' (two 128x128
    # tiles), X (64x64) and beta (64), and writes dQ, dK, dV (three tiles) and dbeta (64 floats)
    tile, st, cc = 64 * 128 * 2, 128 * 128 * 2, 64 * 64 * 2
    want = 6 * tile + 2 * st + cc + 64 * 2 + 3 * tile + 64 * 4
    assert bench.kernel_bytes_per_chunk_head("k_bwd_chunk<bf16,128,128,0>", 128) == want == 221568
    assert bench.kernel_bytes_per_chunk_head("k_bwd_stream<bf16,128,128>", 128) == want - 2 * tile   # no Ut, dUt
    # the specific scan names must not fall through to the plain forward scan's model
    names = ["k_scan_fwd_save", "k_scan_bwd", "k_scan_pair", "k_scan_fwd"]
    assert len({bench.kernel_bytes_per_chunk_head(n, 128) for n in names}) == 4
    # algorithmic bytes per token and head: what the method obliges the pass to move (the layer's tensors, once)
    assert bench.kernel_algorithmic_bytes_per_token_head("k_scan_fwd_save<T, DK, DV, VAR_PLAIN>", 128) == 3 * 256 + 2 + 256 == 1026
    assert bench.kernel_algorithmic_bytes_per_token_head("k_bwd_chunk<T, DK, DV, VAR_PLAIN>", 128) == 4 * 256 + 2 + 3 * 256 + 4 == 1798
    assert bench.kernel_algorithmic_bytes_per_token_head("k_bwd_stream<T, DK, DV>", 128) == 1798
    assert bench.kernel_algorithmic_bytes_per_token_head("k_wy_prep<T, DK, DV>", 128) == 258
    assert bench.kernel_algorithmic_bytes_per_token_head("k_scan_bwd<T, DK, DV, VAR_PLAIN>", 128) == 768
    # model FLOPs per token and head at d = 128: forward 6 d^2 + 10 C d + (2/3) C^2, backward twice the matmul part + 4 C^2
    fwd, bwd = bench.model_flops_per_token_head(128)
    assert abs(fwd - (6 * 16384 + 10 * 8192 + 4096 * 2 / 3)) < 1e-6
    assert bwd == 12 * 16384 + 20 * 8192 + 4 * 4096


def test_measured_traffic_is_read_from_the_tracked_profile_summary():
    # bench.py's `traffic` figures are whatever profiles/hbm_traffic_cfg2_fwd_bwd.txt holds (written by profile_summary.py
    # from the rocprofv3 counter runs), never numbers typed into the script
    sys.path.insert(0, ROOT)
    import bench
    path = os.path.join(ROOT, "profiles", "hbm_traffic_cfg2_fwd_bwd.txt")
    lines = [l.split() for l in open(path) if l.startswith("traffic_bytes ")]
    assert lines, "the summary carries no traffic_bytes lines"
    table = bench.read_measured_traffic()
    assert table == {name: float(val) for _, name, val in lines}
    for need in ("k_wy_prep", "k_scan_fwd_save", "k_scan_bwd", "k_bwd_chunk"):
        assert table[need] > 0
        assert bench.measured_traffic(need + "<T, DK, DV, VAR_PLAIN>") == table[need]
    assert bench.measured_traffic("k_scan_fwd<x>") == table["k_scan_fwd"] != table["k_scan_fwd_save"]
    assert bench.measured_traffic("unknown") is None
    assert bench.read_measured_traffic(os.path.join(ROOT, "profiles", "no_such_file.txt")) == {}
    # and every figure in the table is a plausible per-launch byte count for this workload (between the algorithmic bytes
    # of the smallest kernel and a few times the whole step's)
    assert all(5e7 < v < 3e9 for v in table.values())
