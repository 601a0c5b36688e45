"""Writes loop_tree.json: the 64-node verification tree that the decoding-loop benchmark
uses, as designed by the ORACLE's tree design (section 3.3.1) from the synthetic head
accuracies (5 heads, 10 candidates).  Calls only the oracle and the input generators.
"""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "..", ".."))
from oracle import Oracle  # noqa: E402
from paper_2505_23219_amd import workloads as wl  # noqa: E402

K, R, M = 5, 10, 64
parent, rank, expect = Oracle("f32").tree_build(wl.head_accuracies(K, R), M)
with open(os.path.join(HERE, "loop_tree.json"), "w") as f:
    json.dump({"heads": K, "candidates": R, "nodes": M, "parent": [int(p) for p in parent],
               "rank": [int(r) for r in rank], "expected_acceptance_length": expect}, f, indent=1)
