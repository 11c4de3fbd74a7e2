"""fp64 CPU oracle for the Rodimus DDTS recurrence -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The product path (the HIP library and its
Python binding) never does, and shares no code with it.

Contents
--------
``rodimus_oracle.c``  the sequential recurrence in plain C, IEEE double
                      (paper Sec. 3.1.3, state recurrence of the Rodimus block).
``sequential.py``     ctypes loader for it: ``scan``, ``step``, ``scan_bwd`` (reverse-mode differentiation of the
                      recurrence, step by step), ``block_output`` (feed-through and output gate of Sec. 3.1.3),
                      ``short_conv`` (the ShortConv of Sec. 3.1.3), ``ddts_gates`` (the gate front-end of Sec. 3.1.2) and
                      ``scan_gated`` / ``step_gated`` (the recurrence straight from the gates' pre-activations),
                      ``scan_gated_bwd`` (its backward pass, through the gates and the pre-processing of q and k),
                      ``scan_general`` / ``step_general`` (the general transition of Sec. 3.1.1 with a gate along the value dimension too).
``chunkwise.py``      the same result computed by the chunkwise form of the
                      appendix "Chunkwise Parallel Representation of the Rodimus
                      Block", in numpy fp64 -- used to check the chunk algebra
                      and the chunk-size invariance of the result.
``build.py``          compiles the C file with gcc into ``librodimus_oracle.so``.

Pins (tests/test_oracle_pins.py): reduction to plain causal linear attention,
alpha = 0, the unrolled O(T^2) weighted sum, geometric-series closed form,
a hand-worked rational example, split-sequence and chunk-size invariance;
(tests/test_oracle_backward.py): central finite differences of ``scan``, the
linear-attention closed forms, the T = 1 case by hand, split-sequence chaining;
(tests/test_oracle_backward_gated.py): central finite differences of ``scan_gated``
in every argument (norm guard included), the chain rule against ``scan_bwd`` and
``ddts_gates``, Proposition 1's signs, planted mistakes;
(tests/test_oracle_short_conv.py): hand-worked values, numpy.convolve, impulse
response, identity taps, split-sequence chaining through the carried inputs.
"""
from .sequential import (block_output, ddts_gates, scan, scan_bwd, scan_gated, scan_gated_bwd, scan_general, short_conv,  # noqa: F401
                         step, step_gated, step_general, threads)
