"""MI355X-native BlockPerm-SJLT sketch apply (hand-written HIP behind a C ABI).

The Python layer only marshals arguments; every step of the path runs in the
kernels of libflashsketch.so.  There is no CPU fallback: without the built
library, touching any name of :mod:`paper_2602_06071_amd.binding` raises
ImportError.  (`python -m paper_2602_06071_amd.build` builds it.)
"""

_BINDING_NAMES = {
    "FS_BF16", "FS_F32", "KIND_BLOCKPERM", "KIND_BLOCKROW", "KIND_GAUSS_DENSE", "KIND_SJLT_SCATTER",
    "VARIANT_AUTO", "VARIANT_GENERIC", "VARIANT_MFMA", "FlashSketchError", "Sketch", "lib",
    "lib_path", "fs_info", "SYMBOLS",
}


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
