"""The benchmark's accounting, without a GPU: the algorithmic bytes per GeMM (the numerator of the roofline
fraction) against hand-worked values, and the recorded traffic table."""
import bench
from paper_2310_06178_amd import inputs


def test_algorithmic_bytes_of_the_benchmark_configurations():
    # Section 4.2: m*k weight elements (half a byte each) and k*b activations are read, m*b outputs written;
    # one fp16 scale per 128 weights where the configuration has them
    want = {
        "cfg1": 1024 * 1024 // 2 + 1024 * 4 + 1024 * 4,                                        # 532 480
        "cfg2": 16384 * 4096 // 2 + 4096 * 2 + 16384 * 2,                                      # 33 595 392
        "cfg3a": 14336 * 4096 // 2 + 14336 * 32 * 2 + 4096 * 8 * 2 + 14336 * 8 * 2,            # 30 572 544
        "cfg3b": 14336 * 4096 // 2 + 14336 * 32 * 2 + 4096 * 16 * 2 + 14336 * 16 * 2,
        "cfg4": 8192 * 8192 // 2 + 8192 * 16 * 1 + 8192 * 16 * 4,
        "cfg5": 28672 * 8192 // 2 + 28672 * 64 * 2 + 8192 * 64 * 2 + 28672 * 64 * 2,           # 125 829 120
    }
    assert want["cfg2"] == 33595392 and want["cfg1"] == 532480 and want["cfg3a"] == 30572544 and want["cfg5"] == 125829120
    for name, nbytes in want.items():
        assert bench.algorithmic_bytes(inputs.CONFIGS[name]) == nbytes, name


def test_traffic_table_covers_the_benchmark_configurations():
    for name in ("cfg1", "cfg2", "cfg3a", "cfg3b", "cfg4", "cfg5", "mlp1", "mlp2"):
        nbytes, kernel = bench.measured_traffic(name)
        assert nbytes and kernel, name
        # measured traffic is never below what the method must move, and these kernels stay within 2.1x of it
        alg = bench.algorithmic_bytes(inputs.CONFIGS[name])
        assert alg <= nbytes <= 2.1 * alg, (name, nbytes, alg)
    assert bench.measured_traffic("no such configuration") == (None, None)
