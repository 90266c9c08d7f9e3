"""CPU oracle for the forward 2-D convolution.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It shares no code with the HIP library and never imports it.
"""
from .conv2d_oracle import (  # noqa: F401
    PAD_SAME,
    PAD_VALID,
    build,
    forward_bias_act_f32,
    forward_bias_act_pool_f32,
    forward_f32,
    forward_f64,
    geometry,
    max_pool_2x2,
    max_threads,
    points_f32,
)
