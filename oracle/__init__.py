"""fp64 CPU oracle for the swap-aware training iteration (test infrastructure).

This package is TEST INFRASTRUCTURE ONLY.  It defines what one training
iteration of the transformer stack must compute (plain synchronous minibatch
training, microbatch-major, nothing swapped, nothing recomputed), what the
layer-pack-major schedule of the paper must compute (the same thing), how many
bytes each schedule moves over the host link, and what the balanced-time
packing heuristic returns.  Only the tests, the smoke check and the CPU
baseline leg of the benchmark may import it; the GPU product path never does
and shares no code with it.

Modules
-------
model      the transformer, its backward pass and Adam, in numpy float64
schedule   the layer-pack-major driver (input-batch grouping, recompute,
           jit-compute, jit-update) and the task list it walks
swapcount  closed-form swap volumes and an independent ledger walk
packing    balanced-time packing (Algorithm 2) and the analytic layer profile
"""
