"""CPU oracle for the Lazarus MoE-layer hot path -- TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct NumPy/Python statement of what the path computes,
written from the paper (Lazarus, arXiv 2407.04656) and independent of the HIP
implementation: it shares no code, tables or helpers with `paper_2407_04656_amd/`
and never imports it.  Only `tests/`, `__graft_entry__.smoke()` and the
`cpu_baseline` leg of `bench.py` may import this package; the product path must
never route through it.

Modules
  moe_layer  routing (Sec. 2.1), the token dispatcher (Algorithm 1, Sec. 4.2), the
             per-slot row maps, permute, the expert FFN and the gate-weighted combine
  moe_backward  the layer's backward pass by the chain rule (gradients of inputs, gates,
             logits and expert weights, replica sums as in Sec. 5)
  planner    replica allocation (Eq. 1), MRO / spread placement (Sec. 4.1, Theorem 1),
             recovery probability by enumeration (Sec. 6.3) and re-planning after
             rank loss (Sec. 4.3)

Every function names the passage it follows.  Where the paper is silent, garbled or
ambiguous the reading taken is stated in the docstring.  Pins (tests that tie each
function to something other than itself) live in tests/test_oracle_*.py.

Every function has a pin.  The order and tie rule of the greedy node mapping in
`planner.replan` are a reading (the paper gives no worked example): the implementation of that
reading is pinned by hand-worked cases (tests/golden/replan_handworked.txt) and by an
arg-min check of every pick on random instances.
"""
