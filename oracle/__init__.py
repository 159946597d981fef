"""CPU oracle for the per-layer optimizer step -- test infrastructure, not the product.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It shares no code with ``paper_2512_17570_amd``.
"""
