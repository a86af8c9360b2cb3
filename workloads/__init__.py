"""Seeded synthetic inputs for the Tri-Accel optimizer step.

This package only *generates inputs* (tensor shapes, gradients, probe pairs,
initial parameters, hyper-parameter values).  It contains none of the method's
arithmetic and is the only code shared by the CPU oracle's tests and the HIP
path's tests / benchmark: both sides consume the arrays produced here.

The shapes follow the two architectures the paper trains (Sec. 4, "Setup":
ResNet-18 and EfficientNet-B0 on CIFAR); the value distributions are synthetic
stand-ins for real CIFAR gradients, which need the datasets and trained models.
"""

from .shapes import (  # noqa: F401
    tiny_mlp_shapes,
    resnet18_cifar_shapes,
    efficientnet_b0_shapes,
    large_streaming_shapes,
    mixed_state_shapes,
)
from .configs import Workload, get_workload, WORKLOAD_NAMES, MASTER_SEED  # noqa: F401
