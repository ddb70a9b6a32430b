"""CPU oracle for the mesh-laid-out Transformer-layer einsum path (Mesh-TensorFlow, arXiv 1811.02084).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain, fp64 statement of what the
hot path computes.  Nothing in the product package may import it; only the tests, the
smoke entry and the benchmark's cpu_baseline leg call it.  It shares no code with the
HIP path and never consumes a value produced by it.

Modules
  bf16     round-to-nearest-even to the bfloat16 grid (the storage format of activations)
  einsum   named-dimension einsum by its definition (section "Operation Implementation",
           paragraph "Einstein Summation")
  layout   mesh, computation layout, per-processor slice ("Tensor Representations"),
           lowering of an einsum onto a virtual mesh and its Allreduce groups
  layer    feed-forward and multi-head-attention sublayers of the model-parallel
           Transformer (section 'Model-Parallel "Transformer"'), forward and backward,
           written as sequences of the named einsum
  norm     layer normalisation over d_model (two reductions + component-wise operations),
           forward and backward, alone and after the residual sum
  optim    the step of synchronous data-parallel training with replicated parameters
           (Algorithm 1): sum of the processors' gradients, gradient-descent update; the
           Allreduce point followed by a component-wise operation
  metrics  the error measures the parity tests gate on

Pins (see tests/test_oracle_*.py): brute-force loops on tiny inputs, closed forms
(all-ones), exact integer evaluation, slice shapes and per-processor element counts the
paper prints (worked example and Table 1), the layout-independence statement of the
worked example, Appendix B's two ratios, finite differences and the adjoint identity for
every backward function, closed forms of softmax attention; the error measures of metrics by
hand-computed vectors; the library-backed large-size einsum path against the written-out
definition at sizes where the library re-orders the contraction; layer normalisation by values
worked by hand, closed forms, its shift / scale invariance and finite differences; the training
step by hand-worked values and by the sub-batch gradients adding up to the batch gradient.

Parity unpinned: the layer *semantics* relative to the authors' own Transformer code
(attention scale, mask constant, absence of layer norm / dropout / bias).  The paper
prints no numeric example and defers to external code; the readings taken are listed in
the design notes of this repository.
"""
