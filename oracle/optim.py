"""The step of synchronous data-parallel training with replicated parameters (test infrastructure
only): section "Inspiration: Single-Program-Multiple-Data (SPMD) Batch-Splitting", Algorithm 1.

Each processor computes the parameter gradients of its share of the batch; the gradients are summed
over all processors (the Allreduce) and every processor applies the same update to its copy of the
parameters.  The paper leaves `Update` open; the reading taken is plain gradient descent,
W <- W - lr * (sum of the processors' gradients), on parameters kept in full precision (on the
device: an fp32 master copy), with `store` marking the reduced-precision copy the einsums read.
"""
import numpy as np

from .bf16 import round_to_bf16


def allreduce_sum(grads):
    """Step 2: the sum over processors, in processor order."""
    total = np.zeros_like(np.asarray(grads[0], dtype=np.float64))
    for g in grads:
        total = total + np.asarray(g, dtype=np.float64)
    return total


def sgd_step(master, grads, lr, store=round_to_bf16):
    """Steps 2 and 3 for one parameter tensor: returns (new master copy, the copy the einsums read)."""
    new = np.asarray(master, dtype=np.float64) - lr * allreduce_sum(grads)
    return new, store(new)


def allreduce_then(parts, residual=None, op=None, aux=None, store=round_to_bf16):
    """The point where the partial sums of one group meet (paragraph "Einstein Summation" of
    "Operation Implementation": the Allreduce after the local einsums), optionally followed by a
    component-wise operation on the complete sum (paragraph "Component-wise Operations": no
    communication): residual (if any), then the processors' partial sums in processor order;
    op None: the sum;  op "relu": max(sum, 0);  op "mask": the sum where aux > 0, else 0 (the
    gradient of ReLU, aux being the saved activation).  `store` marks the stored result."""
    total = np.zeros_like(np.asarray(parts[0], dtype=np.float64))
    if residual is not None:
        total = total + np.asarray(residual, dtype=np.float64)
    total = total + allreduce_sum(parts)
    if op == "relu":
        total = np.where(total > 0.0, total, 0.0)
    elif op == "mask":
        total = np.where(np.asarray(aux, dtype=np.float64) > 0.0, total, 0.0)
    elif op is not None:
        raise ValueError(op)
    return store(total)

