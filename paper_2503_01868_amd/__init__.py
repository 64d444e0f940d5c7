"""MI355X-native forward kernels for the Hyena-SE / Hyena-MR gated causal convolutions."""
