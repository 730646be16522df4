"""fp64 CPU oracle of the ReAttention hot path -- test infrastructure only."""
