"""HATA hash-aware top-k decode attention for MI355X (gfx950).

``paper_2506_02572_amd.hata``   ctypes binding of the C-ABI library (HIP kernels)
``paper_2506_02572_amd.synth``  seeded synthetic workload generator (no method arithmetic)

Nothing is loaded at package import; the binding loads ``libhata.so`` on first use
and raises if it is missing or no GPU path can run.
"""
__all__ = ["hata", "synth"]
