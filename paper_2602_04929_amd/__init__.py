"""TurboBoA quantization hot path for MI355X: thin Python binding over the HIP C-ABI library.

`synth` (input generation) imports without the built library; everything else needs
libturboboa.so and raises ImportError when it is missing: there is no fallback path.
"""
from . import synth  # noqa: F401

_BINDING_NAMES = ("Context", "TurboBoAError", "AttnDesc", "LayerDesc", "F32", "BF16", "F64",
                  "GEMM_LOWER", "GEMM_CAUSAL_K", "GEMM_PERSISTENT", "GEMM_A_TILED", "GEMM_B_TILED", "GEMM_C_TILED", "GEMM_F16", "GEMM_KLO", "LIB_PATH")


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding":
        import importlib
        binding = importlib.import_module(__name__ + ".binding")
        return binding if name == "binding" else getattr(binding, name)
    raise AttributeError(name)
