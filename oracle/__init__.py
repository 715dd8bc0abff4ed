"""CPU oracle for the S-STE 2:4 sparse linear layer (arXiv 2409.09099).

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import anything from this package.  The HIP library and
its Python binding never import, link or call it, and it never imports them: the two sides
share no code, tables or constants.

Everything here is plain numpy.  Two layers live side by side:

* a *math layer* in float64 that writes out the definitions of the paper (Sec. 4.1 soft
  threshold, Sec. 4.2 MSE-optimal beta, Sec. 5.1 linear-layer algebra and the MVUE estimator);
* a *bit-spec layer* that replays, in IEEE float32 and integer arithmetic, the exact rounding
  sequence that a storage format (bf16 / OCP e4m3fn, 2-bit position metadata) forces, so that
  masks, metadata and packed values can be compared bit for bit.

Parity status of each function ("pinned" = checked by tests against something other than
itself) is stated in the module headers.
"""
