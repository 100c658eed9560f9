"""AlignedKV decode attention over a precision-aligned KV cache, MI355X (gfx950) native.

The compute path is the HIP library under ``csrc/`` reached through its C ABI
(``include/akv.h``); ``binding`` marshals torch device pointers into it.
"""
