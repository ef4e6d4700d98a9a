"""MI355X-native MoE-offloading decode engine (arXiv 2312.17238): ctypes binding over a HIP library.

`binding` mirrors include/moe_offload.h; `engine.Stack` owns the torch-allocated memory the library
works in.  The HIP library is required: nothing here computes on the CPU.
"""
