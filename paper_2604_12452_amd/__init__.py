"""MI355X-native hot path of Latent-Condensed Attention: liblca (HIP, gfx950) and its thin binding.

``paper_2604_12452_amd.lca``    ctypes binding of the C-ABI library (argument marshalling only)
``paper_2604_12452_amd.inputs`` seeded synthetic inputs (numpy only; shared with the tests' oracle side)
``paper_2604_12452_amd.build``  hipcc driver that compiles csrc/ into liblca.so in-tree
"""
