"""CPU oracle for the dithered-backprop hot path: test infrastructure only.

Nothing in the product package may import this module; see ``oracle.py``.
"""
