"""Float64 CPU oracle for the LongFlow decode step (test infrastructure only)."""
