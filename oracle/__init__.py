"""CPU oracle of the EasyQuant quantization path (test infrastructure only)."""
