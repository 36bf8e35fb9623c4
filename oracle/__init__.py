"""CPU oracle (test infrastructure only; never imported by the product path).

``oracle.forward``  -- plain forward pass of a tenant graph (fp64 accumulation)
``oracle.schedule`` -- segmentation, residue model and granularity-aware search,
                       written step by step from Sections 4.1-4.4
"""
