"""Predictive Pipelined Decoding on one MI355X: Python face of libppd (hand-written HIP behind a C ABI)."""
