"""MI355X-native hot path of TSM video training (temporal shift fused into 2-D
convolutions, BatchNorm/ReLU, residual blocks, the TSM-ResNet-50 train step).

The arithmetic lives in the HIP library under ``csrc/``; ``binding`` only
marshals arguments.  Importing the package does not load the library; calling
any operation without it raises."""
