"""MI355X-native forward path of one ZEDA dynamic-MoE layer (zero-expert injection, Section 2.1)."""
