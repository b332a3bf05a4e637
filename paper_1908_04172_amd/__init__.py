"""MI355X-native RNS-CKKS ciphertext-plaintext MAC + lazy rescale (hot path of arXiv 1908.04172).

`paper_1908_04172_amd.he` is the Python binding of the C-ABI library built from `csrc/`;
`paper_1908_04172_amd.workloads` generates the seeded synthetic layers.
"""
