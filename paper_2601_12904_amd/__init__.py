"""MI355X-native selective-prefill path of FusionRAG (arXiv 2601.12904).

`binding` wraps the C-ABI library built from `csrc/`; `synth` generates seeded inputs.
Importing the package does not load the library; `binding.load()` does and raises if it is missing.
"""
