"""MI355X-native uncollapsed Gibbs sweep (LDA, Gaussian mixture) after Augur, arXiv 1312.3613.

`paper_1312_3613_amd.binding` loads the HIP library (and fails loudly if it is not built);
`paper_1312_3613_amd.synth` draws seeded synthetic inputs and needs no GPU.
"""
__all__ = ["binding", "synth", "build"]
