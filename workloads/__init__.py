"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds shapes, random lengths, allocator op scripts, random values and the
harness's own statement of where an element lives in the pool.  It holds none
of the method's arithmetic and imports neither the oracle nor the library.
"""
