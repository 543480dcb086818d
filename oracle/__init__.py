"""CPU checker (test infrastructure only): see diloco_oracle.py."""
