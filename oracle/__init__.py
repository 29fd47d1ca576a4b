"""CPU oracle (test infrastructure only; see hexa_oracle.cpp)."""
