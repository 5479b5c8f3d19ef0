"""KVzap prune step for MI355X: ctypes binding over the HIP library.

Importing the package loads nothing; `paper_2601_07891_amd.binding` loads the
shared library on first use and raises if it has not been built.
"""
__all__ = ["binding", "synth"]
