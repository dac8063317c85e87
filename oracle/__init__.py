"""CPU oracle of the ScMoE block forward pass: test infrastructure, never a product path."""
