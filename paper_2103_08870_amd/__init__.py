"""MI355X-native compression hot path of Learned Gradient Compression."""
