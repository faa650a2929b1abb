"""CPU oracle for PQTopK scoring: test infrastructure only (tests, smoke check, benchmark CPU-baseline leg)."""
