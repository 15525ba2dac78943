"""Seeded synthetic inputs shared by the CPU oracle and the GPU library.

This package holds *inputs only*: computation graphs (topology + operator
attributes), seeded weight / activation tensors, backend-pattern registries
and seeded integer cost tables.  It contains none of the method's arithmetic
(no operator evaluation, no shape inference, no matching, no search): each
side consumes these descriptions with code of its own.
"""
from .graphdesc import GraphDesc, OP_KINDS                      # noqa: F401
from .models import (tiny_cnn, resnet50, resnext50, bert_base, nasnet_a, resnet3d_50,  # noqa: F401
                     dcgan, random_dag, MODEL_BUILDERS)
from .patterns import (P, W, default_registry, pattern_ops,     # noqa: F401
                       small_registry)
from .costs import synthetic_costs                              # noqa: F401
