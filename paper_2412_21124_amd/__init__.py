"""MI355X-native norm-test statistics pass with fused AdamW (DDP-Norm / FSDP-Norm hot path).

``paper_2412_21124_amd.binding`` is the thin ctypes layer over the C-ABI library
``libnormtest.so`` built from ``csrc/``; ``paper_2412_21124_amd.synth`` draws the
seeded synthetic workloads.  Nothing here falls back to a CPU implementation.
"""
