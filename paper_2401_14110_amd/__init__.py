"""MI355X-native simulated low-bit-width-accumulator (LBA) matrix product.

`paper_2401_14110_amd.binding` is the thin ctypes layer over the C-ABI library built from
`csrc/` (it raises if the library is missing); `paper_2401_14110_amd.inputs` only generates
seeded synthetic operands.  Attribute access below is lazy so that importing the package never
loads the HIP library by itself.
"""

__all__ = ["binding", "inputs"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
