"""MI355X-native Dynamic Vocabulary Pruning hot path.

`paper_2512_23087_amd.dvp` is the thin binding over the C-ABI library built
from `csrc/`; `paper_2512_23087_amd.workloads` holds the seeded input
generators.  Submodules are imported on demand so that the generators can be
used without the compiled library.
"""
