"""CPU oracle of the ZEDA MoE layer: test infrastructure, never imported by the product package."""
