"""MI355X-native training step of the attention-based stacked-LSTM encoder-decoder
(hand-written gfx950 HIP kernels behind a C-ABI library; this package is the thin binding)."""
