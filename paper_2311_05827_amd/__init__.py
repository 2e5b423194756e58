"""MI355X (gfx950) bit-level compressor / decompressor for pipeline-boundary tensors.

The product is libaccept.so (HIP kernels behind a C ABI, see include/accept.h); this
package holds its sources (csrc/), the build step (build.py) and a ctypes binding
(binding.py).  The binding is imported lazily so that ``python -m
paper_2311_05827_amd.build`` works before the library exists.
"""
import importlib

_BINDING_NAMES = (
    "Desc", "make_desc", "AcceptError", "accept_packed_size", "accept_workspace_size", "accept_compress",
    "accept_decompress", "accept_compress_noalloc", "accept_mbq_init", "accept_mbq_compress_first", "accept_compress_timed", "accept_decompress_timed",
    "accept_bits_schedule", "accept_stage_name", "alloc_outputs", "dtype_code", "status_string", "version",
    "UNIFORM", "MBQ", "F32", "BF16", "ROUND_NEAREST_EVEN", "ROUND_STOCHASTIC",
    "LAYOUT_PACKED", "LAYOUT_BATCH", "LAYOUT_UNENCODED",
)


def __getattr__(name):
    if name == "boundary":
        return importlib.import_module(__name__ + ".boundary")
    if name == "binding" or name in _BINDING_NAMES:
        mod = importlib.import_module(__name__ + ".binding")
        return mod if name == "binding" else getattr(mod, name)
    raise AttributeError(name)
