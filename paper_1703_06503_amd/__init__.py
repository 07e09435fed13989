"""MI355X-native auto-tuned SGEMM: a thin Python binding over the C-ABI library."""
