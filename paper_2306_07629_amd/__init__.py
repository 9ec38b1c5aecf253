"""MI355X-native Dense-and-Sparse look-up-table matvec (the inference hot path of SqueezeLLM, Sec. 4.3) and the
offline pass that produces its inputs (Dense-and-Sparse split and sensitivity-weighted k-means, Sec. 4.1-4.2).

The product is ``libsqllm.so`` (hand-written HIP for gfx950, C ABI in ``include/sqllm.h``); this package is
its thin Python binding plus a helper that puts a generated layer on the device."""
from .binding import (SqllmError, lib, sqllm_algorithmic_bytes, sqllm_csr_plan_build, sqllm_csr_plan_bytes, sqllm_csr_spmv, sqllm_csr_spmv_rowwise,  # noqa: F401
                      sqllm_dense_sparse_matvec, sqllm_dense_sparse_matvec_multi, sqllm_multi_launch_order, layer_descriptors, sqllm_dequantize, sqllm_extraction_counts, sqllm_fp16_gemv, sqllm_lut_gemv,
                      sqllm_quantize_layer, sqllm_quantize_layer_noalloc, sqllm_quantize_workspace_bytes, sqllm_unpack_indices, sqllm_version)
from .device_layer import DeviceLayer  # noqa: F401
from .quantizer import QuantizedLayer, quantize_layer  # noqa: F401
