"""CPU oracle for the SwitchBack layer: test infrastructure only (see switchback_oracle.c)."""
