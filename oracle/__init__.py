"""CPU oracle of the GCN hot path: test infrastructure only (see gcn_oracle.cpp)."""
