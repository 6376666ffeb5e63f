"""MI355X-native SK-Net / U-Net hot path (arXiv 1509.03371): Python binding of libsknet.so.

Importing the package does not load the library; `paper_1509_03371_amd.binding` does, and fails
loudly when the built library is missing.
"""
