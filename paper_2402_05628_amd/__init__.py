"""MI355X-native RepQuant inference path (arXiv 2402.05628): thin Python binding over librepquant.so.

Importing the package does not load the HIP library; `paper_2402_05628_amd.binding` does, and fails
loudly when it is missing.
"""
