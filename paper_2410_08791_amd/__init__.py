"""MI355X-native layer-streaming executor (Superpipeline hot path).

`paper_2410_08791_amd.synth` generates the seeded workloads and imports
nothing native; `paper_2410_08791_amd.binding` loads the HIP library and fails
loudly when it has not been built.
"""
