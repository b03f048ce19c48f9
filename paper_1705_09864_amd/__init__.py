"""MI355X-native binary-layer kernels (BMXNet hot path): thin Python binding over libbmx."""
