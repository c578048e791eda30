"""CPU oracle (test infrastructure only): see rom_oracle.py.  Nothing in the product path imports this package."""
