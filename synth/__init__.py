"""Seeded synthetic inputs: tenant operator graphs, weights and input tensors.

This package is data only.  It describes *what* each tenant is (an operator
list in execution order, Section 4.1 "Multi-Tenant Runtime Deployment") and
produces the seeded numbers both the CPU oracle and the GPU library consume.
It contains none of the method's arithmetic: no convolution, no scheduling,
no plan handling.
"""
from .rng import splitmix64_uniform, splitmix64_normal, bf16_round  # noqa: F401
from .graphs import (Op, Tenant, toy_cnn, toy_mlp, resnet18, resnet34, resnet50, resnet101, vgg16,  # noqa: F401
                     alexnet, mobilenetv2, mobilenetv3_large, densenet121, bert_base, small_cnn, small_alexnet,
                     small_mbv2, small_mbv3, small_densenet, small_resnet, small_bert,
                     materialise, gemm_macs, tenant_params)
from .configs import build_config, CONFIG_NAMES  # noqa: F401
