"""Writes tests/golden/shape_grid_200.txt: the 200 (M,N,K) triples of the shape-grid
workload, drawn by workloads.c4_shapes() (seed 1, without replacement).  Calls the input
generators only; run from the repository root:  python tests/golden/make_shape_grid.py"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import workloads  # noqa: E402

path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "shape_grid_200.txt")
with open(path, "w") as f:
    f.write("# 200 distinct (M N K) triples, seed 1, from {64,128,256,512,1024,2048,4096,8192,12288}^3, draw order\n")
    for (m, n, k) in workloads.c4_shapes():
        f.write(f"{m} {n} {k}\n")
print(path)
