"""CPU fp64 oracle for the LAWCAT sequence-mixing path (test infrastructure only)."""
