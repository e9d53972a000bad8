"""CPU oracle package (test infrastructure only; see power_attn_oracle.py)."""
