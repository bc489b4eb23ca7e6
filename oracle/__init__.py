"""CPU oracle of the expert-choice MoE layer: test infrastructure only.

Nothing in the product package may import this; see ec_moe_ref.py.
"""
