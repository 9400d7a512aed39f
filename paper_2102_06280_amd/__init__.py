"""Consensus SGD with dynamic backup workers: one training round for all N simulated
workers on one MI355X, behind a C-ABI library of hand-written HIP kernels.

`inputs` holds seeded synthetic workload generators; `binding` loads the library and
exposes its entry points under the same names.
"""
