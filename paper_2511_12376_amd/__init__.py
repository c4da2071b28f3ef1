"""MI355X-native BitSnap checkpoint codecs: bitmask delta sparsification of 16-bit model states
and cluster quantisation of fp32 optimizer states, as hand-written HIP kernels behind a C ABI.

``paper_2511_12376_amd.synth`` generates seeded inputs and needs no GPU.  The codec entry
points live in ``paper_2511_12376_amd.binding`` and are re-exported lazily here so that the
input generator can be imported on a machine that has no built library.
"""

_BINDING_NAMES = (
    "encode_sparse", "decode_sparse", "quantize_cluster", "dequantize_cluster",
    "sparse_mask_bytes", "sparse_tile_elems", "sparse_workspace_bytes",
    "cluster_param_bytes", "cluster_label_bytes", "cluster_fit_floats", "cluster_workspace_bytes",
    "cluster_z", "version", "lib", "BitsnapError", "debug_stream_copy",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
