"""MI355X-native splatting rasterizer (forward + backward) for point-based differentiable rendering.

`paper_2512_20017_amd.synth`   seeded synthetic scenes (no method arithmetic)
`paper_2512_20017_amd.binding` thin ctypes binding over the C-ABI HIP library (loaded on first use)
"""
__all__ = ["synth", "binding"]
