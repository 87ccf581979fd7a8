"""CPU oracle for the mixed-precision training hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only
tests, the smoke check and the benchmark's cpu_baseline leg may call it.

Model of computation (paper Sec. 3.3 and Sec. 4): tensors are stored in IEEE
binary16; a dot product forms exact FP16xFP16 products, sums them (here in
FP64, standing in for "the exact sum") and rounds ONCE to FP16 on store.  The
optimizer path (Sec. 3.1, 3.2) is a fixed sequence of individually rounded
IEEE FP32 operations on the FP32 master copy.

No code, table or helper is shared with the HIP path.
"""
