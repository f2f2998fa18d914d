"""Seeded synthetic inputs for the SwiftKV prefill path.

This package only *draws inputs* (weights, token ids, prompt lengths, block
tables).  It contains none of the method's arithmetic and is imported by the
tests and the benchmark, which hand the same tensors to the HIP library and to
the CPU oracle.  Neither of those two imports this package or each other.
"""
from .generators import (counter_hash, normal_table, seeded_normal_bf16,
                         seeded_token_ids, seeded_permutation, seeded_uniform01,
                         seeded_fp8_codes)
from .configs import (ModelShape, Workload, WORKLOADS, get_workload,
                      make_weights, WeightStore, build_batch)
