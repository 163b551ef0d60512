"""MI355X-native hot path of the Relation-Aggregation-First HGNN layer (arXiv 2408.09697).

`binding` mirrors the C ABI of include/heta.h one to one; `layer` sequences those calls for a
whole R-GCN-style layer, `rgat` for an R-GAT layer, `sampler` the device sampler for a k-hop
mini-batch, `train` one whole mini-batch training step (sample, forward, backward, Adam).  All computation happens inside libheta.so's HIP kernels.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
from .layer import RafLayer  # noqa: F401
from .rgat import RgatLayer  # noqa: F401
from . import sampler  # noqa: F401
from .train import MiniBatchTrainer  # noqa: F401
