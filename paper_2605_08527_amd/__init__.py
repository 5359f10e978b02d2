"""MI355X-native mixed-tenant multi-LoRA linear layer (C-ABI library + binding)."""
