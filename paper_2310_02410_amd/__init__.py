"""MI355X-native MoQE hot path: top-1-routed MoE expert FFN over int4/int3/int2
weight-only quantized experts (C-ABI HIP library + thin Python binding)."""
