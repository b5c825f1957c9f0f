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


def test_operand_byte_and_flop_models_of_the_dominant_kernel():
    # The roofline's numerator, re-derived by hand for C = 64, d = 128, bf16.  Per (chunk, head) the
    # chunk kernel reads dO, Ut, dUt, K, Q, V (six 64x128 tiles), S and dS' (two 128x128 tiles), X (64x64)
    # and beta (64), and writes dQ, dK, dV (three tiles) and dbeta (64 floats).
    sys.path.insert(0, ROOT)
    import bench
    tile, st, cc = 64 * 128 * 2, 128 * 128 * 2, 64 * 64 * 2
    want = 6 * tile + 2 * st + cc + 64 * 2 + 3 * tile + 64 * 4
    assert bench.kernel_bytes_per_chunk_head("k_bwd_chunk<bf16,128,128,0>", 128) == want == 221568
    # the specific scan names must not fall through to the plain forward scan's model
    names = ["k_scan_fwd_save", "k_scan_bwd", "k_scan_pair", "k_scan_fwd"]
    vals = [bench.kernel_bytes_per_chunk_head(n, 128) for n in names]
    assert len(set(vals)) == 4
    assert bench.measured_traffic("k_scan_fwd_save<x>") == bench.MEASURED_HBM_BYTES["k_scan_fwd_save"]
    assert bench.measured_traffic("k_scan_fwd<x>") == bench.MEASURED_HBM_BYTES["k_scan_fwd"]
    assert bench.measured_traffic("unknown") is None
    # model FLOPs per token and head at d = 128: forward 6 d^2 + 10 C d + (2/3) C^2, backward twice the matmul part + 4 C^2
    fwd, bwd = bench.model_flops_per_token_head(128)
    assert abs(fwd - (6 * 16384 + 10 * 8192 + 4096 * 2 / 3)) < 1e-6
    assert bwd == 12 * 16384 + 20 * 8192 + 4 * 4096
