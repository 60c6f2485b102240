"""TEST INFRASTRUCTURE ONLY: plain, slow CPU statements of what the GPU library computes.

Nothing in the product imports this package; only ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py`` do.  Nothing here imports the GPU package.
"""
