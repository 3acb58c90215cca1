"""MI355X-native cache-gated transformer layer (LLMCache hot path).

``workloads`` draws seeded synthetic inputs; ``llmc`` is the thin binding over
the C-ABI library ``libllmc.so`` (loaded lazily, on first use).
"""
