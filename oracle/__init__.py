"""CPU oracle of the ProphetKV hot path: test infrastructure only.

Nothing in the product package may import this; see ``pkv_oracle``.
"""
