"""MI355X-native server-side linear layers of GALA (arXiv 2105.01827)."""
