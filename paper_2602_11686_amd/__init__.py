"""MI355X-native MoE-layer hot path (gate, permute, grouped SwiGLU FFN fwd/bwd, combine).

``binding`` mirrors the C ABI of include/moe.h; ``layer`` owns the buffers and
the call order; ``inputs`` holds the seeded synthetic workloads.
"""
