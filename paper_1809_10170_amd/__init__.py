"""MI355X-native direct convolution (forward, fp32, zero workspace).

`workloads` (shapes + seeded inputs) imports without a GPU; the binding in
`conv_direct` loads the HIP shared library on first use and raises if it is missing.
"""
