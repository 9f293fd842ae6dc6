"""TurboBoA quantization hot path for MI355X: thin Python binding over the HIP C-ABI library."""
