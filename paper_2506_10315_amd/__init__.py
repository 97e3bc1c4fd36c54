"""MI355X-native learned-optimizer step (small_fc_lopt, VeLO): thin binding over liblopt.so.

Every step of the optimizer runs in the HIP kernels behind the C boundary of include/lopt.h;
this package only marshals arguments. There is no CPU fallback: if the library is not built,
loading it raises.
"""
from .binding import (LoptError, LearnedOptimizer, lib, lopt_config, lopt_tensor_desc,  # noqa: F401
                      default_config, weights_count, LOPT_SMALL_FC, LOPT_VELO)


def __getattr__(name):
    # the torch.optim veneer imports torch at module level; load it on first use only
    if name == "LearnedOptTorch":
        from .optim import LearnedOptTorch
        return LearnedOptTorch
    raise AttributeError(name)
