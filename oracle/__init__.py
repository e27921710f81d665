"""CPU oracle for the layout-elided transformer chains (SmartMem, arxiv 2404.13528).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) imports, links or calls anything in this package, and this
package imports nothing from the product.  Only tests/, the smoke check and the
benchmark's cpu_baseline leg use it.

Everything is numpy float64 (integer work is int64).  Every layout
transformation (Reshape, Transpose/Permute, cyclic roll, window partition and
reverse, head split and merge, patch merging, NCHW<->token rearrangement) is
materialised as a new contiguous array: this is the explicit chain that the
paper's elimination (Sec. 3.2.1) must reproduce exactly, because layout
transformations are pure data movement.

Pins (tests marked "not gpu"): the paper's Tables 3, 5, 6, the worked examples
of Sec. 2.2 and Sec. 3.2.2 (Fig. 4), brute force on tiny tensors, algebraic
identities, and torch CPU library routines as an independent third opinion.
The paper prints no numeric block outputs, so block values beyond those pins
are "parity unpinned" with respect to the paper itself.
"""
