"""CPU oracle of the ROCKET transform (paper section 3, Eq. 1-4).

TEST INFRASTRUCTURE ONLY.  Slow, plain and independent of the HIP library:
only tests, the smoke check and the benchmark's cpu_baseline leg import it.
"""
from .sampler import sample_kernel, sample_kernels  # noqa: F401
from .ridge import ridge_fit, ridge_predict  # noqa: F401
from .prologue import znormalize_u8  # noqa: F401
from .train import feature_matrix, mse_loss_grad, sgd_update, loss_of, train_step  # noqa: F401
from .minirocket import minirocket_kernels, minirocket_fit_bias, minirocket_transform  # noqa: F401
from .rocket_oracle import (  # noqa: F401
    conv_output, transform, backward, num_threads, set_threads, AMBIGUOUS_EPS,
)
