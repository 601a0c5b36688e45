"""Writes workload_trees.json: the parent[] arrays of the named workloads.

These are inputs (tree shapes), not expected outputs; the file pins them so a
change in the random-number library cannot silently change the workloads.
Calls only the input generators.
"""
import json
import os
import sys

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", ".."))
from paper_2505_23219_amd import workloads as wl  # noqa: E402

out = {name: [int(p) for p in wl.workload(name).parent]
       for name in ("tiny", "layer7b", "stack7b", "stack13b")}
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "workload_trees.json"), "w") as f:
    json.dump(out, f, indent=1)
