"""CPU oracle (test infrastructure only; see nezha_oracle.cpp)."""
