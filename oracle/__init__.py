"""CPU oracle of the RAF HGNN layer.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the product path (`paper_2408_09697_amd`) never does, and this package
imports nothing from it.  Edge loops live in `heta_oracle.c` (plain C, fp64
accumulation, explicit edge lists); dense steps are numpy fp64 matmuls; the sparse
optimizer step of the learnable tables is in `optim.py`; graph attention as the
relation-specific aggregation (R-GAT) is in `rgat.py`; k-hop neighbour sampling into blocks
is in `sampler.py`; meta-partitioning of the metagraph is in `metapartition.py`.
"""
from .optim import sparse_adam_step
from . import rgat
from . import sampler
from . import metapartition
from .layer import (aggregate_bwd, aggregate_fwd, aggregate_fwd_f32_sequential, build, csc, cross_rel_sum, in_degree,
                    layer_backward, layer_forward, project, project_bwd, LayerResult)

__all__ = ["aggregate_bwd", "aggregate_fwd", "aggregate_fwd_f32_sequential", "build", "csc", "cross_rel_sum", "in_degree",
           "layer_backward", "layer_forward", "project", "project_bwd", "LayerResult", "sparse_adam_step", "rgat", "sampler",
           "metapartition"]
