"""MI355X-native forward pass of one pipeline stage (prefill and decode phases).

Importing the package does not load the HIP library; `paper_2506_10470_amd.tdp`
does, and fails loudly when it has not been built.
"""
