"""CPU oracle for the linear-algebraic data-movement primitives and the
partitioned layers built from them (Hewett & Grady, arXiv 2006.03108).

This package is TEST INFRASTRUCTURE.  It is a plain, slow, fp64 numpy
transcription of what the paper defines; it shares no code with the HIP
library and must never be imported by the product path.  Only the test
suite, the smoke check and the CPU-baseline leg of the benchmark use it.

Modules
  memory_model  Sec. 2: allocate / deallocate / clear / add / copy / move as
                explicit block matrices.
  geometry      Sec. 3 "Halo exchange" + App. B.1: balanced splits, output
                index ranges, halo / pad / extra widths per worker.
  primitives    Sec. 3: broadcast, sum-reduce, all-reduce, scatter / gather,
                nested halo exchange H and its adjoint H*, the adjoint test.
  layers        Sec. 4: convolution, affine and pooling, both as the plain
                (sequential) definition and as the paper's distributed
                algorithms; the point-wise / loss glue of the Sec. 5 network.

Parity pins: every function here is checked in tests/ (run with -m "not gpu")
against values the paper prints (App. B.1 examples, App. C table), against
closed forms, brute force, and independent library routines.
"""
