"""CPU oracle for the ODMA decode hot path -- TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct implementation of what the GPU library
computes: single-query GQA softmax attention over per-request KV held in
contiguous slabs / paged blocks / dense padding (``oracle.attention``), and a
step-by-step simulation of the ODMA bucket allocator with its Large-Bucket
safety pool and histogram recalibration (``oracle.allocator``).

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package.  It shares no code with the HIP path and never imports
it; the product path must not route through anything here.
"""
