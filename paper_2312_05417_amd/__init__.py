"""MI355X-native re-ranking hot path of multi-vector (late-interaction) retrieval:
candidate gather through CSR offsets, MaxSim scoring (Eq. 1, Sec. 2.1) and ranked top-k,
as hand-written HIP for gfx950 behind a C-ABI library.

`paper_2312_05417_amd.binding` loads the built library (and fails loudly when it is
missing); `paper_2312_05417_amd.synth` draws the seeded synthetic inputs.  Importing this
package loads neither.
"""
__all__ = ["binding", "synth"]
