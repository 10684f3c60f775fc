"""AKVQ-VL KV-cache hot path for AMD MI355X (gfx950): 2-bit write path and decode attention.

`paper_2501_15021_amd.synth`   seeded synthetic workloads (no method arithmetic)
`paper_2501_15021_amd.binding` thin ctypes binding of the C-ABI library (libakvq.so, hand-written HIP)
"""
__all__ = ["synth", "binding"]
