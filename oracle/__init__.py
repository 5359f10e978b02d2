"""fp64 CPU oracle (test infrastructure only; see lora_oracle.c)."""
