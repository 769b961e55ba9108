"""CPU fp64 oracle for prefix-shared attention (BatchLLM, Sec. 4.3.3 and Sec. 5).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) may import this package; only the tests, the smoke check and the
benchmark's cpu_baseline leg use it.  It shares no code with the HIP path.

Parity status of each function:
  attention.attend_one, attention.prefix_shared_attention  -- pinned to the plain
      definition softmax(q K^T / sqrt(d)) V by brute force with a dense mask, by
      a stock fp64 scaled-dot-product-attention routine, by closed forms and by
      metamorphic invariants (tests/test_oracle_*.py).
  attention.lse_merge  -- pinned by "split anywhere + merge == unsplit",
      associativity/commutativity, identity of the empty part.
  packing.pack_token_batch  -- pinned by hand-written expected arrays under
      tests/golden/ and by structural invariants.
  Numeric parity with values printed in the paper: unpinned (the paper prints no
  attention value; its kernel comparison exists only as a figure).
"""
