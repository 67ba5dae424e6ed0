"""MI355X-native Gradient Alignment Control (GAC) step: C-ABI library + thin binding.

Nothing is loaded at import time; ``paper_2603_01501_amd.binding`` opens the HIP
library on first use and raises if it is not built.
"""
