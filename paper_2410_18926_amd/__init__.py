"""MI355X-native query phase of LoRANN (reduced-rank-regression ANN search): HIP library + thin binding.

`paper_2410_18926_amd.binding` wraps the C-ABI library (`include/lorann.h`); `paper_2410_18926_amd.synth`
makes the seeded synthetic corpora, queries and index arrays.  Importing the package does not load the HIP
library; `binding` raises if it has not been built.
"""
__version__ = "0.1.0"
