"""KVBuffer-style Gated DeltaNet decoding for AMD MI355X (gfx950).

``kvb``      ctypes binding of the C-ABI library (kvb_decode / kvb_flush /
             kvb_verify / kvb_direct); loads libkvb.so on first use and raises if
             it has not been built.
``synth``    seeded synthetic workloads.
``traffic``  algorithmic HBM byte counts per call (the roofline denominators).
"""
__all__ = ["kvb", "synth", "traffic"]
