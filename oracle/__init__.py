"""CPU oracle for the deduplicated prefill forward pass.

TEST INFRASTRUCTURE ONLY.  Nothing here is part of the product path: only ``tests/``,
``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may import it.  It shares
no code with the HIP library and imports nothing from the ``paper_2601_15013_amd`` package.
"""
