"""Host-side checks that need no GPU: the benchmark's contract for more than one GPU, the seeded generator's
reproducibility and structure, and that nothing on the product path imports the oracle."""
import os
import re
import subprocess
import sys

import numpy as np

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_product_path_never_imports_the_oracle():
    # only tests/, the smoke check and bench.py's cpu_baseline leg may touch oracle/
    pkg = os.path.join(ROOT, "paper_2411_02886_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), f
                assert "tokenselect_oracle" not in text, f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    uses = [m.start() for m in re.finditer(r"^\s*import oracle\b", bench, flags=re.M)]
    assert len(uses) == 1 and bench.rfind("def ", 0, uses[0]) == bench.find("def cpu_baseline")
    assert "import oracle" not in open(os.path.join(ROOT, "workloads.py")).read()


def test_generator_is_reproducible_and_structured():
    a = W.make_workload("g", dtype=W.BF16, B=2, H=8, H_kv=2, D=64, P=16, seq_lens=[300, 45], k=16, beta=2.5,
                        planted_per_head=3, seed=11)
    b = W.make_workload("g", dtype=W.BF16, B=2, H=8, H_kv=2, D=64, P=16, seq_lens=[300, 45], k=16, beta=2.5,
                        planted_per_head=3, seed=11)
    assert np.array_equal(a.k_pool, b.k_pool) and np.array_equal(a.q, b.q) and np.array_equal(a.page_indices, b.page_indices)
    c = W.make_workload("g", dtype=W.BF16, B=2, H=8, H_kv=2, D=64, P=16, seq_lens=[300, 45], k=16, beta=2.5,
                        planted_per_head=3, seed=12)
    assert not np.array_equal(a.k_pool, c.k_pool)
    # page table: CSR, every sequence owns distinct physical pages, enough for its length
    assert a.page_indptr[0] == 0 and len(a.page_indptr) == 3
    pages = [a.pages_of(i) for i in range(2)]
    assert len(pages[0]) >= (300 + 15) // 16 and len(pages[1]) >= (45 + 15) // 16
    allp = np.concatenate(pages)
    assert len(set(allp.tolist())) == len(allp)
    # planted tokens: per query head, inside the sequence, distinct
    for bi, n in enumerate([300, 45]):
        pl = a.planted[bi]
        assert pl.shape == (8, 3) and pl.min() >= 0 and pl.max() < n
    # bf16 storage: values survive a round trip through float32 exactly
    f = W.as_f32(a.k_pool, W.BF16)
    assert np.array_equal(W.store(f, W.BF16), a.k_pool)


def test_configurations_have_the_shapes_the_benchmark_names():
    w = W.config1()
    assert (w.dtype, w.H, w.H_kv, w.D, w.P, w.k, int(w.seq_lens[0])) == (W.F32, 8, 2, 64, 16, 256, 4096)
    lens = W.config3_lengths()
    assert len(lens) == 8 and lens.min() >= 16384 and lens.max() <= 65536
    w5 = W.config5(N=2048, C=32)
    assert w5.C == 32 and int(w5.seq_lens[0]) == 2048 + 32 and w5.extra["n_cached"] == 2048
