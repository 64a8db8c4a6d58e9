"""CPU oracle (test infrastructure only): see ffn24_oracle.py."""
