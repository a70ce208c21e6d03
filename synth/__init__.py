"""Seeded synthetic inputs and layer shapes shared by the tests, the benchmark
and the oracle's callers.

This module holds no arithmetic of the method: it only draws tensors of the
shapes and value distributions of the workloads (ResNet-style convolution
layers with value-independent synthetic data; the paper's own runs use layer
shapes of VGG16/ResNet18/ResNet50 with untrained or all-ones data, Sec. 5.2 and
Sec. 5.4) and names the layer shapes.  Random numbers come from
numpy.random.Generator(PCG64(seed)); activations are drawn first, filters second.
"""
from .shapes import ConvShape, CONFIG1, CONFIG2, CONFIG3, CONFIG4, resnet50_layers
from .gen import (int8_tensors, fp16_tensors, ones_tensors, requant_params, seed_for)

__all__ = ["ConvShape", "CONFIG1", "CONFIG2", "CONFIG3", "CONFIG4", "resnet50_layers",
           "int8_tensors", "fp16_tensors", "ones_tensors", "requant_params", "seed_for"]
