"""MI355X-native fused Multi-Head FFN (FlashMHF hot path).

`paper_2512_06989_amd.mhffn` is the thin binding over the C-ABI library built
from `csrc/`; `paper_2512_06989_amd.inputs` draws the seeded synthetic
workloads.  Nothing is loaded at import time."""
