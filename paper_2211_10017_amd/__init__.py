"""MI355X-native sparsely activated expert FFN layer with weight-only int4/int8 experts.

The work is done by the HIP library behind ``include/moe_wq.h``; ``binding`` marshals torch
device pointers into its C entry points (loaded on first use, and failing loudly if the
library has not been built).  ``workloads`` holds the seeded synthetic input generators.
"""
