"""fp64 CPU oracle for the SVGD all-particle update (test infrastructure only)."""
