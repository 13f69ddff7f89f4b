"""MI355X-native MMSE INT4 scale search (arXiv 1902.06822, Sections 3.3-3.5, 3.7).

``binding`` wraps the C ABI of ``libmmse_hip.so`` (hand-written gfx950 kernels);
``synth`` draws the seeded CNN-shaped workloads; ``select`` holds the host-side
key-layer rule.  The binding imports torch; ``synth`` and ``select`` do not.
"""
__all__ = ["synth", "select"]
