"""Seeded synthetic inputs (IDs, offsets, gradients, table values).

Shared by the CPU oracle's tests and the HIP path's tests and bench; holds none
of the embedding layer's arithmetic and imports neither of them.
"""
from .workloads import (BASE_SEED, BF16, F32, MEAN, SUM, Batch, FieldSpec, TableSpec, Workload,
                        bf16_bits_to_f32, build_cpu, build_hip, config, fill_device, make_batch,
                        make_batches, mix64, split_batch, table_rows)
