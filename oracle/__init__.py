"""fp64 CPU oracle of the SLA forward -- test infrastructure only (see sla_oracle.c)."""
