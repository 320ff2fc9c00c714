"""MI355X-native learner hot path of Parallel Q-Learning (PQL).

``workloads`` draws the seeded synthetic inputs; ``binding`` is the thin ctypes layer over
the C-ABI library ``libpql.so`` (HIP kernels for gfx950) built from ``csrc/``.
"""
