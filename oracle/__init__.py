"""CPU oracle for the Global-QSGD hot path (test infrastructure only; see gq_oracle.c)."""
