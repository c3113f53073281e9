"""MI355X-native decode attention operator (the attention-worker hot path of
model-attention disaggregation, paper Sec. 2.1 / 2.2.2 / 4.2.2).

``paper_2405_01814_amd.lamina`` is the thin ctypes binding over the C-ABI HIP library;
``paper_2405_01814_amd.workloads`` draws the seeded synthetic batches.  Nothing here
falls back to a CPU implementation: using the binding without the built library raises.
"""
