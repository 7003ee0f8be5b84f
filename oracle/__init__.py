"""CPU oracle for the data-parallel hot path of Synkhronos (arXiv 1710.04162).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package:
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg use it.
It shares no code with the HIP library and never imports it.

Everything here is plain NumPy in float64 (or exact integer work), written as
the definition of what each step of the path computes:

  split       Sec. 3.2 "Function Calling" step 1 (inputs scattered equally, as
              possible, over workers) and Sec. 5.1 (a worker's share is cut
              into slices the same way); Sec. 4.1 (first tensor dimension =
              independent data points).
  gather      Sec. 5.2 (a list of row indexes selects the minibatch; each
              worker excerpts its own contiguous share of the list).
  mlp         the "function" of Sec. 2 / Sec. 3.3 step 1: loss and gradient of
              a ReLU MLP with softmax cross-entropy on a set of rows, the
              sliced/aggregated evaluation of Sec. 5.1 and the worker reduce of
              Sec. 3.2 step 3.
  convblock   a second such function: a 3x3 convolution + batch-normalisation
              block with the ending of the scaling study's network (Sec. 6),
              evaluated per slice the same way.
  reduce      Sec. 3.1 "Build Functions" (a reduce/gather op per output),
              Sec. 3.3 step 2 (all-reduce of the flat gradient).
  collectives Sec. 3.2 "Shared Variable Management" (broadcast, all-reduce,
              all-gather over the N worker copies), App. A (parameter average).
  update      Sec. 3.3 step 3 (the update rule applied with the combined
              gradient on the flat parameter array: momentum, Nesterov
              momentum, RMSProp, Adam).
  evalops     a six-output evaluation function, each output with its own
              reduce op, aggregated over slices (Sec. 3.1, Sec. 5.1).
  brute       pure-Python-loop twins used only to pin the NumPy code at tiny
              sizes.

Pins (tests/test_oracle_*.py): finite differences, closed forms, brute-force
loops, library routines (np.array_split, np.take, scipy logsumexp,
torch.optim.SGD / RMSprop / Adam on CPU where the formulas coincide,
hand-worked single elements where they do not, torch.bfloat16 casts) and the paper's defining
invariant (Sec. 1.1): aggregating independent calls over any subdivision of
the data equals the one full-batch call.

The bfloat16 modes (mlp.function and convblock.function with bf16_points=True) are
pinned too: a scalar-loop twin with its own rounding routine (brute.py) for the MLP,
torch autograd with rounded operands for the block, each with negative cases in which
one rounding point is dropped, added or moved.  No function here is unpinned.
"""
