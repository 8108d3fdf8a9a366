"""CPU oracle of the LiteAttention hot path -- test infrastructure only (see lite_attn_oracle.c)."""
