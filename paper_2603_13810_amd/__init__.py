"""MI355X-native forward path of Temporal Aggregated Convolution (TAC / TAC-TP).

``paper_2603_13810_amd.api`` is the thin binding over the C-ABI library
(``libtac.so``, hand-written HIP for gfx950); ``paper_2603_13810_amd.synth``
holds the seeded synthetic workloads.  Importing the package loads nothing
native; the first call into ``api`` loads the library and fails loudly if it
has not been built.
"""
__all__ = ["api", "synth"]
