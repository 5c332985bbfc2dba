"""CPU oracle (test infrastructure only; see at_grpo_oracle.py)."""
