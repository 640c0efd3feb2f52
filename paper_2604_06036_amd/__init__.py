"""MI355X-native codec-guided sliding-window prefill hot path (CodecSight, arXiv 2604.06036).

Importing the package loads nothing heavy; the HIP library is opened on first use of
`paper_2604_06036_amd.binding` and a missing library is an error, never a CPU fallback.
"""
__all__ = ["binding", "planner", "synth", "engine"]
