"""CPU oracle (test infrastructure). See linattn_oracle.c for what it defines."""
