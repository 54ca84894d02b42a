"""MI355X-native SpeCache decode-step hot path (arXiv 2503.16163).

`paper_2503_16163_amd.binding` loads the HIP library and exposes the C-ABI
calls under the same names; `paper_2503_16163_amd.synth` draws the seeded
synthetic inputs.  Importing the package itself loads nothing.
"""
