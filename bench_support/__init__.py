"""Measurement yardsticks used by bench.py only: a small HIP library of its own
(libbench_probes.so, built from bench_probes.hip), kept apart from libcp_attn."""
