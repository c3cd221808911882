"""CPU oracle for the delta-serving linear layer -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package; the
product path (the HIP library and its binding) never does, and this package never imports them.

Two independent writings of the same definition (paper Section 5.1 Eq. (2), Section 5.2):
  * `c`  -- oracle/dz_oracle.c through ctypes: plain loops, fp32 (or fp64) accumulation in
            ascending k; this is the oracle parity tests compare the GPU against, and the one
            the benchmark times on the host cores;
  * `np_` -- oracle/np_oracle.py: numpy fancy indexing + a library matmul, used to cross-check
            the C one.
"""
from . import c_oracle as c          # noqa: F401
from . import np_oracle as np_       # noqa: F401
from . import lora_oracle as lora    # noqa: F401   (low-rank adapters: Section 3.2, Section 6.4)
from . import compress_oracle as compress_   # noqa: F401   (data-free 2:4 + RTN compressor: Section 4.1 steps 2-3)
from . import quant_oracle as quant    # noqa: F401   (quantisation-only deltas, merged weights: Section 4.1 step 3, Section 5.1 Eq. (2))
