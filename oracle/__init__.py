"""CPU oracle for the breadth-first / depth-first training step.

TEST INFRASTRUCTURE ONLY.  Plain numpy in float64, written from the paper
(arXiv 2211.05953) and from the textbook definitions of the transformer layer
it trains.  Nothing in the product package may import this; only tests, the
smoke check and the cpu_baseline leg of the benchmark do.  It shares no code,
table or constant with the HIP path.

Modules
  layer     one pre-LN GPT transformer layer, forward and hand-derived backward
  stack     a rank's N_loop stages run in BF or DF order, main-grad
            accumulation, Adam, integer event trace
  schedule  unit-time pipeline simulator for N_PP >= 1 (bubble, checkpoints)
  formulas  the paper's closed forms (App. A)

Pin status: every function is pinned by tests under tests/ marked "not gpu"
(finite differences, torch autograd, brute force, closed forms, the paper's
printed worked values).  End-to-end activations/gradients are not printed by
the paper, so no golden tensors exist: for those, finite differences, the
autograd cross-check and the BF == DF == one-big-batch invariants are the pins.
"""
