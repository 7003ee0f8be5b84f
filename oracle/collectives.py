"""The collectives over the N worker copies of a variable (Sec. 3.2, the part
on shared variables, which lists broadcast and all-reduce among its
collectives; App. A: averaging the parameters over workers; Sec. 3.2 step 3:
results reduced or gathered).  With the workers emulated as N buffers, each
collective maps a list of N arrays to a list of N arrays:

  broadcast    every worker receives the root's array
  all_reduce   every worker receives the reduction (in list order) of all N
               arrays with the given op; op "mean" with weights omega_w = 1/N
               is the parameter / gradient average
  all_gather   every worker receives the concatenation of all N arrays in
               worker order (the arrays may differ in length)

reduce-to-one and gather-to-one are reduce.reduce_buffers itself.
"""
import numpy as np

from .reduce import reduce_buffers


def broadcast(src, n_workers):
    src = np.asarray(src)
    return [src.copy() for _ in range(n_workers)]


def all_reduce(bufs, op, weights=None):
    if op == "concat":
        raise ValueError("all_reduce takes an arithmetic op; use all_gather")
    r = reduce_buffers(bufs, op, weights)
    return [r.copy() for _ in bufs]


def all_gather(bufs):
    c = reduce_buffers(bufs, "concat")
    return [c.copy() for _ in bufs]
