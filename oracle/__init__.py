"""CPU oracle of the PLAID search path -- test infrastructure only (see plaid_oracle.c)."""
