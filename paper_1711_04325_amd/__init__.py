"""MI355X-native ResNet-50 training-step kernels (librn50.so) and their thin Python binding."""
