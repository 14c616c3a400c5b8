"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU library's tests and benchmark."""
from .workloads import (CTX8K, CTX16K, CTX32K, PAPER32K, STACK32K, TINY, WORKLOADS, Workload, bf16_bits, confidence,
                        layer_qkv, masked_all, shared_direction, strong_sinks)

__all__ = ["CTX8K", "CTX16K", "CTX32K", "PAPER32K", "STACK32K", "TINY", "WORKLOADS", "Workload", "bf16_bits", "confidence",
           "layer_qkv", "masked_all", "shared_direction", "strong_sinks"]
