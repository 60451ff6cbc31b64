"""MI355X-native hot path of PaSS (parallel speculative sampling): the (1+k)-token decode step.

Importing the package loads nothing heavy; `paper_2311_13581_amd.binding` loads the HIP library.
"""
__all__ = ["synth"]
