"""MI355X-native Log-linear Sparse Attention (forward + backward of one layer).

``paper_2512_16615_amd.llsa`` is the ctypes binding of the C-ABI library built
from ``csrc/``; ``paper_2512_16615_amd.inputs`` holds the seeded workload
generators.  Nothing is loaded at import time.
"""
