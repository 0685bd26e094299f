"""MI355X-native mixed-precision quantized linears (the hot path of LLM-PQ, arXiv 2403.01136)."""
