"""MI355X-native convolution block (vl_nnconv) of the MatConvNet manual: forward and backward."""
