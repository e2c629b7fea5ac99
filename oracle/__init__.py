"""CPU oracle of the Ladder-Residual shard forward: test infrastructure, never on the product path."""
