"""MI355X-native AutoAssist hot path: Assistant score -> Bernoulli keep -> stable
compaction -> gather -> hinge-loss SGD step on the kept rows -> Assistant update.

The work is done by hand-written HIP kernels for gfx950 behind a C-ABI library
(include/autoassist.h).  `paper_1905_03381_amd.api` is the thin ctypes binding;
`paper_1905_03381_amd.synth` draws the seeded synthetic inputs.
"""
__all__ = ["api", "synth", "build"]
