"""CPU oracle for the fused-RoPE paged-attention path — TEST INFRASTRUCTURE ONLY.

Nothing in the product package may import this. Only `tests/`, `__graft_entry__.smoke()` and the
`cpu_baseline` leg of `bench.py` call it. It shares no code with the HIP library.

  oracle.attn   fp64 attention (plain C + OpenMP in mepic_oracle.c, loaded through ctypes)
  oracle.align  the chunk-to-page aligner and pool accounting in plain Python
  oracle.commit the commit step (scatter of new K/V into pages, fp8 quantisation) in numpy
"""
