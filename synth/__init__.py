"""Seeded synthetic inputs (weights, caches, token ids, draft shapes).

This package is the only code shared by the CPU oracle's tests and the GPU
harness.  It contains no arithmetic of the verification method: only
reproducible pseudo-random inputs and the shape tables of the workloads.
"""
from .rng import normal_f32, normal_bf16, uniform_i32, uniform_f64, bf16_bits_to_f32
from .workload import (ModelShape, TINY, LLAMA8B, LLAMA70B, MINI_BF16, WeightSource,
                       WORKLOADS, Workload, make_requests, synthetic_kv, page_lists,
                       tree_parents, stream_id)
