"""CPU fp64 oracle for the block randomized SVD hot path.  TEST INFRASTRUCTURE ONLY:
imported by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg; the
product path (paper_1706_07191_amd) never imports it and shares no code with it."""
