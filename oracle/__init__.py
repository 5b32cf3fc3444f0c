"""CPU oracle of the reassembled low-bit linear layer.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package.  It shares nothing with ``paper_2310_08041_amd`` and never imports it.
"""
