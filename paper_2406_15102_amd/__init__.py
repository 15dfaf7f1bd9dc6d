"""MI355X-native HLQ backward pass (arXiv 2406.15102): thin Python binding over the C-ABI HIP library."""
