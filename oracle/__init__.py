"""CPU oracle for the RPS lossy-averaging round (test infrastructure only)."""
