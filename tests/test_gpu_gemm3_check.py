"""The direct-load GEMM core in its bounds-checking build (tests/native/gemm3_check.hip): every direct load is
tested against the address range of the operands, and the results against fp64 sums of small-integer inputs.
Shapes: the triangular multiply, the fused update and the products with k-slow operands at the sizes of the benchmark configurations whose kernels
these are (C3, C4 r=1024, C5 classes), plus small ones that exercise one and two operand pairs."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "gemm3_check")

CASES = [
    ("nt", 16384, 1024, 1, 3),     # C4 r=1024: rows of Z, rank, triangular factor, three split-bf16 pairs
    ("nt", 8192, 2048, 1, 3),      # C3
    ("nt", 4096, 512, 0, 1),
    ("nt", 4096, 512, 0, 2),
    ("nt", 8192, 2048, 1, 3, 1),   # C3 again, 128-wide column tiles visited from the costliest down
    ("nt", 16384, 1024, 1, 1, 1),
    ("nt", 16384, 2048, 1, 3, 2),  # 512 tiles of 256 x 256 (two rounds), costliest column tiles first
    ("k5", 2048, 4096, 2048, 0, 0),
    ("k5", 3072, 8192, 768, 6, 1),  # a C5 class, column groups of 6 tiles, streaming epilogue
    ("k5", 8192, 3072, 2048, 2, 0),
    ("k5", 2048, 4096, 2048, 3, 1),  # groups of 3 tile columns: 32 columns leave a ragged last group
    ("k5", 3072, 8192, 512, 10, 1),
    ("k5", 1024, 1024, 512, 3, 0),
    # operands with k as the slow index (transposing LDS reads): M N K aks bks nseg lower splitk tail
    ("ks", 53248, 1024, 16384, 1, 1, 1, 0, 1, 1),   # C4 r=1024, the product with (M+G)^T: 832 tiles, the last 64 split over k
    ("ks", 16384, 1024, 53248, 0, 1, 1, 0, 1, 0),   # C4 r=1024, the product with Q (row-major bf16 Q as the right operand)
    ("ks", 2048, 2048, 8192, 1, 1, 3, 1, 6, 0),     # C3 Gram matrix: three operand pairs, lower tiles, six splits over the rows
    ("ks", 768, 768, 3072, 1, 1, 3, 1, 1, 0),       # a C5 class Gram matrix
    ("ks", 8192, 768, 3072, 1, 1, 1, 0, 1, 0),
    ("ks", 3072, 768, 8192, 0, 1, 1, 0, 1, 0),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_direct_loads_stay_in_bounds_and_results_match(case):
    if not os.path.exists(EXE):
        pytest.fail("tests/native/gemm3_check is not built: run python -m paper_2504_05295_amd.build")
    print("running", case, flush=True)
    p = subprocess.run([EXE] + [str(x) for x in case], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=110)
    print(p.stdout, flush=True)
    assert "violations 0" in p.stdout
    assert " bad 0" in p.stdout
    assert p.returncode == 0
