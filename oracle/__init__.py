"""CPU oracle for the Clebsch-Gordan tensor product and its fused graph convolution.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its Python
binding, the planner) imports, links or calls anything in this package, and nothing in
this package imports the product.  The only callers are the test-suite, the smoke check
and the CPU-baseline leg of the benchmark.

Everything here is the plain definition evaluated in fp64 with numpy:

  irreps.py  irreps strings, segment offsets, path enumeration       (paper Sec. 2.1, 2.4)
  cg.py      Clebsch-Gordan blocks: Racah closed form -> real basis   (paper Sec. 2.2-2.3)
  so3.py     real spherical harmonics, Wigner D matrices              (paper Sec. 2.1)
  tp.py      TP(P, x, y, W) of Eq. 1, its gradients (Sec. 3.3)        (paper Eq. 1, Sec. 3.3)
  conv.py    CSR construction, graph convolution of Eq. 4, gradients  (paper Sec. 3.5)

Parity pins (what each function is checked against, apart from itself) live in
tests/test_oracle_*.py.  Functions whose output cannot be pinned to anything but a
convention of ours say "parity unpinned" in their docstring.
"""
