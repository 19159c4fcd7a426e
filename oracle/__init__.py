"""CPU oracle of the SV hot path: test infrastructure only (see sv_oracle)."""
