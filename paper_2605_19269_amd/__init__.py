"""MI355X-native GEMM-plus-epilogue library (Python side: argument marshalling only)."""
