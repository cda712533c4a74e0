"""MI355X-native Top-k + error-feedback gradient compression (GraVAC hot path)."""
