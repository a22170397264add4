"""Plain fp64 CPU oracle of the fused transformer-layer training step.

TEST INFRASTRUCTURE ONLY. Nothing in the product package may import this; it exists so that the
HIP path can be checked element by element against an obviously correct, unfused, slow definition.
It shares no code with the HIP path.
"""
