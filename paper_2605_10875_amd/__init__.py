"""MI355X-native action-conditioned decoder-layer forward pass (SOL hot path).

`paper_2605_10875_amd.sol` is the Python binding of the C-ABI library built from `csrc/`;
`paper_2605_10875_amd.synth` holds the seeded input generators. Importing the package is
cheap; the HIP library is loaded on first use and its absence is an error, never a fallback.
"""
__all__ = ["synth", "sol"]
