"""CHOCO-Gossip / CHOCO-SGD step for all n workers on one MI355X (gfx950).

The compute lives in the HIP shared library built from csrc/; `binding`
marshals arguments into its C ABI and raises if the library is missing.
`synth` makes seeded synthetic inputs and has no dependency on the library.
"""
__all__ = ["binding", "synth", "build"]
