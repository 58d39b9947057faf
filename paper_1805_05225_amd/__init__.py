"""MI355X-native masked LSTM / BLSTM layer (forward + BPTT) behind a C ABI.

`paper_1805_05225_amd.binding` is the thin ctypes layer over the HIP library;
`paper_1805_05225_amd.synth` draws the seeded synthetic benchmark inputs.
"""
