"""CPU oracle for the MoE-instance layer step of Janus (arXiv 2512.13525).

TEST INFRASTRUCTURE ONLY.  A plain, slow NumPy / pure-Python statement of what the
hot path computes, written from the paper.  It shares no code with the HIP
library and is imported only by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  The product path never calls it.

  gating.py      the router's linear layer (gate logits from the activations)  (Sec. 3.3)
  routing.py     gating selection: top-k ids and normalised weights        (Sec. 3.4, Step 0)
  scheduling.py  replica layout tables and Alg. 1 (AEBS), plus the two
                 comparison policies the evaluation describes              (Sec. 3.4, Alg. 1; Sec. 5)
  optimum.py     exact min-max optimum of the scheduling problem           (Sec. 3.4 problem statement)
  dispatch.py    this instance's share of Step 4 (permute) and the
                 weighted top-k combine                                     (Sec. 3.3, Sec. 3.4)
  ffn.py         grouped SwiGLU expert FFN and the dense per-token layer   (Sec. 2.2 roofline paragraph)
  placement_opt.py  window statistics, replica counts, Alg. 3 placement   (Appendix B)
  scaling.py     latency model, steady-state batch, Alg. 2                  (Sec. 3.5)
  bounds.py      balls-into-bins expectation and a_max bound               (Appendix A, Eq. 4-5)

Floating point is fp64 unless a decision must be taken in the kernel's fp32
(see routing.route_sigmoid_group).  Every function is pinned by tests under
tests/ marked "not gpu"; none is "parity unpinned".
"""
