"""MI355X-native denoise-step path for masked-diffusion LLM decoding (lazy-loading package)."""
