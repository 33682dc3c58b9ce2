"""CPU oracle for SparseDrop's fused block-dropout GEMMs (test infrastructure only)."""
