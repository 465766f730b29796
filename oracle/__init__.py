"""CPU oracle of the LIME inference hot path: test infrastructure only.

Nothing in the product package may import this; see lime_oracle.py.
"""
