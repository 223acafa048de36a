"""Seeded synthetic inputs shaped like the paper's workloads.

This module only makes data (design matrices, labels, starting points, run
parameters).  It holds none of the method's arithmetic: no gradients, no
quantizer, no prox.  Both the CPU oracle's tests and the HIP library's tests
and benchmark draw their inputs from here so that they see identical bytes.

The paper's own datasets (its synthetic regression sets, YearPredictionMSD,
MNIST, CIFAR-10, ILSVRC-12) are not available; the five configurations below
stand in for them: dense Gaussian designs at the paper's feature scale, a
sparse text-like design, a correlated ridge design for the accelerated
variant, and a small MLP for "deep model, whole-gradient quantization".
"""
from .configs import SynthProblem, make, CONFIG_NAMES, gaussian_u  # noqa: F401
