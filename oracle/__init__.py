"""CPU oracle for the stacked-RNN forward pass (test infrastructure, not part of the product)."""
