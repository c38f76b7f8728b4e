"""MI355X-native secure-layer hot path of MPC-Pipe's online phase (two parties, Z_2^64).

``paper_2209_13643_amd.mpc``   ctypes binding over the C-ABI library (HIP kernels, gfx950)
``paper_2209_13643_amd.synth`` seeded synthetic inputs (no protocol arithmetic)
"""
__all__ = ["synth"]
