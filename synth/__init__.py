"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package draws random tensors and rounds them to the storage type.  It holds
none of the method's arithmetic (no attention, no entropy, no head, no accept
rule): both sides receive the same bits and compute on their own.
"""
