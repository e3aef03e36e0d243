"""CPU oracle for the HiF8 conversion path (test infrastructure only)."""
