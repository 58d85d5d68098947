"""MI355X-native ring-step kernels for Striped Attention (arxiv 2311.09431).

The compute lives in a C-ABI shared library built from the HIP sources under
csrc/ (see include/striped_attn.h).  `paper_2311_09431_amd.binding` marshals
torch device pointers into it; nothing here computes on the CPU.
"""
