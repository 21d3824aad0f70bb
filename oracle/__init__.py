"""CPU oracle (test infrastructure).  See cb_oracle.c for what it states and cb_oracle.py for the loader."""
