"""CPU oracle of the tree-verification step: test infrastructure only (see s4c_oracle.h)."""
