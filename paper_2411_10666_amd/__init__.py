"""Batched suffix-automaton draft retrieval for AMD gfx950 (arxiv 2411.10666).

``paper_2411_10666_amd.binding`` is the Python face of the C ABI in
``include/sam.h`` and loads the compiled HIP library; ``synth`` draws the seeded
synthetic workloads.  Importing the package itself loads nothing.
"""
