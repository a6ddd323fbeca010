"""MI355X-native hybrid delta attention (DeltaLLM, arXiv 2507.19608): C-ABI library + thin binding."""
