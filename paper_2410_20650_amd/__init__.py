"""MI355X-native NeuZip hot path: bf16 exponent rANS codec behind a C ABI."""
