"""MI355X-native hot path of intra-GPU prefill/decode disaggregation (one mixed-batch
transformer step on disjoint compute-unit partitions).  `binding` wraps the C-ABI
library built from `csrc/`; `synth` holds the seeded input generators."""
