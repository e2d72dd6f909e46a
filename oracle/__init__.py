"""CPU oracle of the multi-LoRA layer: test infrastructure, never a product code path."""
