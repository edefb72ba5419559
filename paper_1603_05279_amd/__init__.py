"""MI355X-native XNOR-Net binary convolution (forward path)."""
