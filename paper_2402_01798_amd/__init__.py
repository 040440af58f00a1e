"""Truncated quantization of heavy-tailed gradients (arXiv 2402.01798) on MI355X.

``binding``  thin ctypes layer over the C-ABI library ``libtq.so`` (HIP, gfx950)
``synth``    seeded synthetic heavy-tailed gradients for tests and benchmarks
"""
