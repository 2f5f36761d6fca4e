"""CPU oracle of the mixed-precision MoE block: test infrastructure, not the product."""
