"""MI355X-native hot path of the CCL-D decision analyzer (cross-rank anomaly
analysis of collective-communication traces).

`paper_2605_04478_amd.ccld` is the binding of the HIP library; it is imported
on first use so that the input generators can be used without it.
"""
__all__ = ["tracegen"]
