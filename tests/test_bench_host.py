"""Host-side accounting of the benchmark: algorithmic bytes, additions of the network a kernel runs, and the
counter-based traffic table that bench.py reads (no GPU work)."""
import importlib.util
import os

from paper_1610_06209_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_algorithmic_bytes_are_x_once_and_output_once_at_every_size():
    c = W.CONFIGS
    assert W.algorithmic_bytes_per_vector(c["cfg1_plain_n256"]) == 2 * 1024
    assert W.algorithmic_bytes_per_vector(c["cfg2_lsh_n1024"]) == 4096 + 64
    assert W.algorithmic_bytes_per_vector(c["cfg3_rff_n4096"]) == 48 * 1024
    assert W.algorithmic_bytes_per_vector(c["cfg4_jl_n16384"]) == 68 * 1024
    assert W.algorithmic_bytes_per_vector(c["cfg5_large_n2p20"]) == 8 << 20          # not the 32 B/element of the schedule
    assert W.schedule_bytes_per_vector(c["cfg5_large_n2p20"]) == 32 << 20
    for k in range(10, 21):
        w = W.sweep_workload(k)
        assert W.algorithmic_bytes_per_vector(w) == 8 << k
        assert W.schedule_bytes_per_vector(w) == (8 << k if k <= 16 else 32 << k)
    blocks = W.NEXT["next_blocks_n4096_L4"]
    assert W.algorithmic_bytes_per_vector(blocks) == 4 * 4096 + 4 * 8 * 4096


def test_additions_count_the_network_that_runs():
    c = W.CONFIGS
    assert W.adds_per_vector(c["cfg1_plain_n256"]) == 3 * 8 * 256
    assert W.adds_per_vector(c["cfg2_lsh_n1024"]) == 16 * 3 * 10 * 1024
    assert W.adds_per_vector(c["cfg3_rff_n4096"]) == 3 * 12 * 4096
    # first 1024 of 16384: two full rounds, then sums over the four highest index bits and ten stages on 1024 values
    assert W.adds_per_vector(c["cfg4_jl_n16384"]) == 2 * 14 * 16384 + 15360 + 10 * 1024 == 484352
    assert W.adds_per_vector(c["cfg5_large_n2p20"]) == 3 * 20 * (1 << 20)


def test_traffic_table_rows_are_found_by_workload_and_form():
    b = _bench()
    t = b.measured_traffic_bytes("sweep_plain_n2p12", "signs")
    assert isinstance(t, int) and abs(t / (8 << 28) - 1.0) < 0.01
    assert isinstance(b.measured_traffic_bytes("cfg5_large_n2p20", "signs"), int)
    assert b.measured_traffic_bytes("sweep_plain_n2p12", "no such form") is None
    assert b.measured_traffic_bytes("no such workload", "signs") is None
