"""CPU oracle (test infrastructure only): see tempo_oracle.c / tempo_oracle.py."""
