"""MI355X-native block-selective mixed-precision attention (ThriftAttention, arXiv 2605.23081).

``binding`` wraps the C ABI of the HIP library (include/thrift.h); ``workloads`` draws the seeded
synthetic inputs; ``metrics`` holds the evaluation arithmetic.  Nothing is loaded at import time:
the HIP library is opened on first use and its absence is an error, never a fallback.
"""
__all__ = ["binding", "workloads", "metrics", "build"]
