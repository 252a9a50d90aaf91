"""OAPL trainer-step loss head for MI355X (gfx950): HIP kernels behind a C ABI.

``paper_2602_19362_amd.oapl`` binds the shared library; ``synth`` draws seeded
synthetic rollout batches.  Importing the package does not load the library;
calling into ``oapl`` without a built library raises.
"""
