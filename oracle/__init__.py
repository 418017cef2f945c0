"""CPU oracle of the Fira optimizer step.  Test infrastructure: see fira_oracle.py."""
