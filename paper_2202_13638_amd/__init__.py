"""MI355X-native batched rollouts through pathwise-sampled GP dynamics (arXiv 2202.13638).

``synth``   seeded synthetic workloads (inputs only; importable without a GPU)
``binding`` thin ctypes binding over the C-ABI library ``libbagel.so`` (HIP, gfx950)
"""
