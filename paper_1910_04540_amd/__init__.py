"""MI355X-native low-precision quantization kernels (fixed point, custom float, block floating
point, fused quantized SGD step) behind the ``libqsim`` C-ABI.

``binding`` marshals torch tensors into the C-ABI; ``workloads`` draws the synthetic inputs.
"""
