"""MI355X-native noisy-channel autoencoder hot path: thin Python binding over libaemodel.so.

Importing the package does not load the library; paper_2602_17681_amd.binding does, and it
raises if the HIP library has not been built (there is no CPU fallback).
"""
