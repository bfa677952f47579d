"""CPU oracle of the KVCapsule hot path: test infrastructure, never on the product path."""
