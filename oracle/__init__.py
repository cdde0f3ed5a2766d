"""CPU oracle for the quantised Winograd/Toom-Cook convolution in the Legendre base.

TEST INFRASTRUCTURE ONLY.  Everything under this package is a plain, slow,
step-by-step CPU statement of what the method computes (exact ``Fraction``
matrices, int64 integer stages, fp64 real arithmetic, and an ``np.float32``
emulation of the single-multiply requantisation).  It shares no code with the
HIP library and must never be imported by the product package; only the test
suite, the smoke check and the benchmark's CPU-baseline leg may call it.

Parity status of each part (what pins it besides itself):

* ``matrices``      pinned: printed P^T / P^{-T} (Section 4.1), non-zero counts,
                    monic Legendre recurrence, exact identity with brute-force
                    correlation, multiplication counts (Sections 1-2).
* ``direct``        pinned: it *is* the textbook definition; cross-checked
                    against scipy.signal.correlate2d.
* ``winograd``      pinned: eq. 3 / eq. 4 equal direct correlation exactly in
                    rational arithmetic and to 1e-10 in fp64.
* ``quantised`` integer stages   pinned by brute force on tiny inputs, by the
                    inner_quant=0 identity (Legendre == canonical bit for bit),
                    by exact-rational rounding, and by an a-priori error bound.
* ``flex``          (run-time fp32 matrices, Section 4.2) pinned where fp32 is exact
                    (must equal ``quantised`` bit for bit), by scalar loops on one
                    tile, and by convergence to an fp64 evaluation of eq. 3 / eq. 4
                    with the same arbitrary matrices; outputs for trained
                    matrices: **parity unpinned** (none are published).
* ``backward``      (gradients of one layer, straight-through casts) pinned: with
                    unquantised operands it must equal the gradients of direct
                    convolution written from the definition; adjoint identities
                    against the forward oracle; exact finite differences; scalar
                    loops; the flex part (gradients of the trained matrices) also
                    by finite differences of an unquantised flex forward pass.
                    The treatment of a cast in the backward pass is a reading
                    (the paper gives none).
* ``quantised`` absolute output values: **parity unpinned** by the paper (it
                    prints no worked numeric example; its quantisation figure is
                    missing).  They are pinned oracle <-> GPU only.
"""
