"""MI355X-native implementation of METok's token-compression hot path.

``synth`` (seeded inputs) imports nothing from the HIP binding; the binding is
loaded on first use of ``paper_2506_02850_amd.binding`` and fails loudly when the
compiled library is missing.
"""
