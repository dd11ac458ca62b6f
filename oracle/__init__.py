"""CPU oracle for the tiled GPT-2 block (test infrastructure, not product code).

Plain numpy, fp64, written from the paper's statement of the operations
(section 3) and, where the paper is silent, from the readings listed in the
design notes.  Two modules:

  definition.py  the untiled definition of every operation, the block forward,
                 its analytic adjoint, the Adam and SGD-with-momentum steps,
                 the embedding layer and the cross-entropy loss.  Tiling only
                 regroups sums, so this is what any tiled execution must
                 reproduce.
  tiled.py       the same operations carried out tile by tile in the order the
                 paper describes (products and sums of elementary tiles for the
                 linear layer, three steps for layer norm, two subroutines for
                 softmax), and attention walked key tile by key tile with the
                 softmax subroutines' running statistics, with its recomputing
                 adjoint.  It exists to pin tiling invariance.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It shares no code with the HIP library and never calls it.
Every function is pinned by tests that do not go through the oracle itself
(brute force, closed forms, finite differences, library routines); none is
"parity unpinned".
"""
