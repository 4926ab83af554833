"""MI355X-native inverse of a causally masked convolution and its backpropagation."""
