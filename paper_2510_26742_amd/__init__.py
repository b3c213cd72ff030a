"""MI355X-native pi0 forward pass (arXiv 2510.26742 hot path).

`synth` holds the seeded input generators; `binding` loads the HIP library and
exposes its C entry points under the same names.  Importing the package loads
nothing heavy: the shared library is opened on first use of `binding`.
"""
