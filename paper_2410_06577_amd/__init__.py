"""MI355X-native hot path of the Rodimus DDTS gated linear-attention recurrence.

``rodimus``    thin ctypes binding of the C-ABI library built from ``csrc/`` (HIP, gfx950):
               ``chunk_scan_fwd`` and ``decode_step``.  Argument marshalling only.
``workloads``  seeded synthetic inputs shaped like the paper's layers.

The binding loads the HIP library on first use and raises if it is missing:
there is no CPU fallback.
"""
__all__ = ["rodimus", "workloads"]
