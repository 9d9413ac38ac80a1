"""CPU oracle of the MoC FFN hot path: test infrastructure, never imported by the product."""
