"""The byte-accounting convention (32-bit items, CSR theta) is the paper's Table 1."""
import bench


def test_table1_flops_per_byte(golden):
    rows = {r[0]: r for r in golden("table1_flops_per_byte.txt")}
    acc = bench.paper_unshared_accounting(k_d=37, k=1000)
    ratios = []
    for step, (flops, nbytes) in acc.items():
        _, f, ints, floats, printed = rows[step]
        per_item = int(f) / (4 * (int(ints) + int(floats)))
        assert abs(flops / nbytes - per_item) < 1e-12          # independent of K_d and K
        assert abs(round(flops / nbytes, 2) - float(printed)) <= 0.005 + 1e-9
        ratios.append(flops / nbytes)
    assert round(sum(ratios) / 4, 2) == float(rows["average"][4])
    # the paper's unshared accounting per token: 32 K_d + 24 K bytes
    assert sum(b for _, b in acc.values()) == 32 * 37 + 24 * 1000


def test_bench_refuses_more_than_one_gpu():
    """`bench.py --gpus N` with N above 1, or a multi-rank launch, ends with a message before
    anything touches a GPU."""
    import os
    import subprocess
    import sys
    here = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for argv, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "2"})):
        p = subprocess.run([sys.executable, os.path.join(here, "bench.py"), *argv], capture_output=True,
                           text=True, env={**os.environ, **env}, timeout=120)
        assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout == ""
