"""fp64 CPU oracle of the per-stage training step.  Test infrastructure: never imported by the product path."""
