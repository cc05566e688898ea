"""MI355X-native PowerSGD+ compressor hot path (arXiv 2509.11254).

`paper_2509_11254_amd.psgd` is the thin binding over the C-ABI library built from `csrc/`;
`paper_2509_11254_amd.synth` draws the seeded synthetic inputs.  Importing the package does not
load the GPU library; `psgd` loads it on first use and fails loudly when it has not been built.
"""
