"""CPU oracle of the DyMoE mixed-precision MoE layer.

Test infrastructure only: nothing in the product package may import this.
"""
