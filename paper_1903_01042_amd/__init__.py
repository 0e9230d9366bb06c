"""MI355X-native CodeNet coded layer step: Python binding over the C-ABI HIP library."""
