"""CPU oracle for the interleaved-ZeRO reshard + snapshot/checksum path.

TEST INFRASTRUCTURE ONLY.  Nothing under this package is part of the product:
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
it.  It shares no code with the HIP library (no kernels, headers, helpers,
tables or constants) and imports nothing from the product package.

Everything here is plain numpy / pure Python, written from the definitions in
the paper (ElasWave, arXiv 2510.00606):

  layout.py    per-unit uniform ("interleaved") ZeRO partition (Sec. 6.3,
               "Interleaved Assignment"; Fig. 10b), ring snapshot placement
               (Sec. 5.1), reconstruction of the logical flat state and its
               re-slicing at a new DP degree (Sec. 5.2 "Live Remap"; Sec. 6.3
               closing paragraph: a pure ownership-layout transformation),
               and the per-(holder -> destination) message contents that the
               overlap matrix M_overlap of Fig. 7b stands for.
  brute.py     the same maps, one element at a time, by scanning; tiny sizes.
  checksum.py  per-1-MiB-block wrapping-u64 sum and XOR of the little-endian
               64-bit words ("online verification", abstract), and the
               bad-block set of a verification pass.

Every function is pinned by tests/test_oracle_*.py against something other
than itself (the paper's D=4, F={2} scenario, closed forms, library routines
in special cases, brute force).  No function here is "parity unpinned".
"""
