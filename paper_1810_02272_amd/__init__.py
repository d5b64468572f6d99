"""MI355X-native Caffe-semantics convolution and InnerProduct layers and policy-gradient loss kernels (fp32): thin Python binding over libmi355conv.so.

The package holds the HIP sources (``csrc/``), the build step (``build.py``), the ctypes binding
(``binding.py``: same names as the C entry points, argument marshalling only) and the seeded
synthetic workloads (``workloads.py``).  There is no CPU fallback: without the built library, or
without a GPU for the compute calls, the binding raises.
"""
from .binding import (  # noqa: F401
    ConvError,
    ConvParams,
    conv_backward_bias,
    conv_backward_bias_f64,
    conv_backward_data_f64,
    conv_backward_filter_f64,
    conv_desc_kernel_names_f64,
    conv_desc_workspace_bytes_f64,
    conv_forward_f64,
    conv_backward_data,
    conv_backward_filter,
    conv_backward_filter_bias,
    conv_backward_filter_static,
    conv_static_workspace_limit,
    conv_desc_create,
    conv_desc_destroy,
    conv_desc_kernel_names,
    conv_desc_output_shape,
    conv_desc_workspace_bytes,
    conv_forward,
    conv_status_string,
    library_path,
)
from .ip_binding import (  # noqa: F401
    IpParams,
    ip_backward_bias,
    ip_backward_data,
    ip_backward_filter,
    ip_desc_create,
    ip_desc_destroy,
    ip_desc_kernel_names,
    ip_desc_workspace_bytes,
    ip_forward,
    ip_relu_backward,
)
from .pg_binding import (  # noqa: F401
    pg_discount_rewards,
    pg_sigmoid_bottom_diff,
    pg_sigmoid_sample_action,
    pg_softmax_bottom_diff,
)
