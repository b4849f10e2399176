"""CPU oracle for the OPT-Tree decoding-step hot path (arxiv 2406.17276).

TEST INFRASTRUCTURE ONLY.  Everything in this package is a plain, slow, fp64
NumPy restatement of what the method computes, written from the paper.  It is
imported by the test-suite, by the smoke check and by the benchmark's
"cpu_baseline" leg -- never by the product path, and it imports nothing from
the HIP package.

  opt_tree.py        draft-tree construction (Sec. 3: Eq. 1-3, Thm. 3.1/3.2,
                     Algorithm 1 with a fixed number of drafting steps)
  tree_attention.py  tree-masked attention used by the verification forward
                     (Sec. 3, Algorithm 2: the mask that goes with the tree)

Parity pins (tests/test_oracle_*.py, marker "not gpu"):
  row statistics      -> scipy.special.logsumexp, closed form for constant rows,
                         brute-force Python sort for the top-k order
  greedy tree         -> exhaustive enumeration of every ancestor-closed
                         n-subset of tiny k-ary universes (definition of E_sub),
                         a hand-derived worked example (tests/golden/),
                         Thm. 3.1 (closure), Thm. 3.2 (monotone E_sub), special
                         cases n=1, k=1, n >= pool
  mask / positions    -> walking parent[] to the root; popcount == depth
  tree attention      -> chain tree == textbook causal attention, gather form
                         (dense attention over prefix+ancestors only), star
                         tree, relabelling equivariance, GQA == replicated MHA,
                         constant-V
Nothing the paper reports numerically (tables, figures) can pin this path: they
depend on trained models and datasets; for those: parity unpinned.
"""
