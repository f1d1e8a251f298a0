"""MI355X-native pipeline-stage F/B/W engine (HIP kernels behind a C ABI)."""
