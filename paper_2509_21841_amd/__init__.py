"""MI355X-native attention engine over packed variable-length sequences (Zeppelin's single-GPU hot path).

`binding` wraps the C ABI of libzeppelin_attn.so; `synth` holds the seeded input generators.
"""
