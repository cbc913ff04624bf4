"""MI355X-native full-batch GLM training iteration (the data-parallel hot path of
the iterative ML jobs that a quality-driven scheduler allocates resources to).

``glm``   : Python binding of the C-ABI library (argument marshalling only).
``synth`` : seeded synthetic input generators.
"""
__all__ = ["glm", "synth"]
