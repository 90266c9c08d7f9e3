"""MI355X-native forward 2-D convolution (NHWC input, HWCF filter, NHWC output).

The compute lives in a C-ABI HIP library (csrc/, declared in include/conv2d.h);
`binding` marshals torch device pointers into it.  `workloads` holds the
synthetic layer shapes and seeded input generators.
"""
