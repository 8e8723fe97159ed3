"""MI355X-native fused LSTM / deep BLSTM forward + BPTT (HIP kernels behind a C ABI)."""
