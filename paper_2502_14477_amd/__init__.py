"""MI355X-native hot path of Efficient Selective Attention (ESA, arXiv 2502.14477).

The work is done by hand-written HIP kernels in libesa.so (C ABI, include/esa.h); this package
is the thin Python binding over it.  There is no CPU or PyTorch fallback: touching any binding
name without the built library raises ImportError.  The binding is loaded on first use so that
`python -m paper_2502_14477_amd.build` can run before the library exists.
"""
_BINDING_NAMES = (
    "ESA_F32", "ESA_BF16", "ESA_W_ROWMAJOR", "ESA_W_PACKED", "ESA_SPLIT_I_EARLY", "ESA_SPLIT_ALGORITHM1", "EsaError", "PackedWeights", "EXPORTS", "lib", "lib_path",
    "esa_version", "esa_segments", "esa_pack_weights", "esa_compress", "esa_score", "esa_select_topk", "esa_gather_kv", "esa_attend", "esa_attend_local", "esa_attend_finish", "esa_attend_indexed", "esa_rope", "esa_attend_reencoded", "esa_compress_qk",
    "esa_select_topk_static", "esa_select_topk_static_capacity", "esa_select_topk_static_prepare", "esa_score_select_gather",
)
__all__ = list(_BINDING_NAMES)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
