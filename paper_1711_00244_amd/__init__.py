"""MI355X-native inference from pruned, codebook-quantised, Huffman-coded layers.

``binding`` mirrors the C ABI declared in include/compressed_layer.h;
``workloads`` draws the seeded synthetic inputs.  The HIP library is loaded on
first use and there is no CPU fallback.
"""
from .binding import (PATH_AUTO, STATIC_SCRATCH_BYTES, PATH_MFMA_BF16, PATH_MFMA_F32, PATH_SPARSE, PATH_SPARSE_WIDE, CLError, Layer, LayerGroup, compress_layer,  # noqa: F401
                      compressed_conv_forward, compressed_fc_forward, compressed_fc_forward_static, compressed_fc_stack_forward, conv_block_h, conv_workspace_bytes, decode_layer,
                      fc_resolved_path, fc_stack_workspace_bytes, fc_workspace_bytes, layer_deserialize, lrn_forward, maxpool_forward, plan_batches)
