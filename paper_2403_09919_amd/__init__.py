"""MI355X-native ReDrafter verification step (dedup -> tree attention -> accept).

`synth` holds the seeded workload generators; the HIP library binding is loaded
on first use of `paper_2403_09919_amd.binding` (it raises if the library is not built).
"""
__all__ = ["synth"]
