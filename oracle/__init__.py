"""CPU oracle for the Gated Sparse Attention (GSA) forward path.

TEST INFRASTRUCTURE ONLY.  Nothing under this package is part of the product:
it is a plain, slow, fp64 restatement of the paper's equations that the GPU
library is checked against.  Only the tests, the smoke check and the
``cpu_baseline`` leg of the benchmark may import it.  It shares no code with
the HIP path and never imports the GPU package.

Modules
-------
gsa_oracle   numpy fp64, one function per stage (Sec. 3.3-3.6) + dense brute force (Eq. 2)
naive        pure-Python loops for tiny cases (second, independent statement)

Parity status: every function is pinned by ``tests/test_oracle_pins.py``.
"""
