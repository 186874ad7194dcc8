"""CPU oracle for the paged-decode hot path.

TEST INFRASTRUCTURE ONLY.  Nothing under this package is part of the product:
it may be imported by the tests, by the smoke check and by the benchmark's
CPU-baseline leg, and by nothing else.  It shares no code with the HIP
library or its Python binding, and imports neither.

  alloc.py  two-level (LCM) page allocator with request-aware placement,
            plus the per-request page lists that become block tables
            (paper Sec. 4.1, 4.3; sliding-window need set of Sec. 5.1).
  attn.py   dense masked softmax attention over contiguous K/V in fp64
            (the textbook definition; the window of Sec. 5.1, Fig. last-access).
  attn_threads.py  the same computation in fp32 on a thread pool: a second, faster CPU
            figure for the benchmark's report, pinned against attn.py; never the reference.
"""
