"""MI355X-native fused latent -> frame decoder (HIP kernels behind a C ABI)."""
