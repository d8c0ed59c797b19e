"""CPU oracle (test infrastructure).  See slowmo_oracle.py / slowmo_oracle.c."""
