"""MI355X-native LAWCAT prefill path: causal depthwise Conv1D -> normalized gated linear attention."""
