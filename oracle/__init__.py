"""CPU oracle of the batch-SOM epoch: test infrastructure, never on the product path."""
