"""fp64 CPU oracle of the MSLA module -- test infrastructure only (see msla_oracle.c)."""
