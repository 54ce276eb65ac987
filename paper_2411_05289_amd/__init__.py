"""MI355X-native sampling-verification for multi-draft speculative decoding
(SpecHub, RRS, RRSw).  The compute lives in the HIP library under ``csrc/``;
``binding`` marshals torch tensors into its C ABI."""
