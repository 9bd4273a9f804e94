"""LASP-2 hot path (chunked causal linear attention, forward + backward) for MI355X.

The arithmetic lives in the HIP library `liblasp2.so` (see csrc/ and
include/lasp2.h); `binding` marshals arguments to its C ABI.
"""
