"""MI355X-native chunked low-precision classifier head (ELMO, arxiv 2510.11168)."""
