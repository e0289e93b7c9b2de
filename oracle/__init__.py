"""CPU oracle (test infrastructure only; never imported by the HIP package)."""
