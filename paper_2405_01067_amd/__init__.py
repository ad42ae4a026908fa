"""MI355X-native hot path of AB-training (arxiv 2405.01067): factored-layer forward/backward
and the factor merge, as hand-written HIP kernels behind a C-ABI library."""
