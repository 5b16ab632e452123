"""MI355X-native per-block Shampoo optimizer step (C-ABI HIP library + thin binding)."""
