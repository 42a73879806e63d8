"""CPU oracle of the LLSA layer: test infrastructure only (never imported by the GPU package)."""
