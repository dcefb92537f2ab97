"""MI355X-native fused sparse-linear attention (SLA): C-ABI HIP library + thin Python binding."""
