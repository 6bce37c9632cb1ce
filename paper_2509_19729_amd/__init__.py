"""MI355X-native reshard of a running instance's state from TP=k to TP=k'.

The compute lives in hand-written HIP kernels behind a C-ABI library
(``include/amoeba.h``); :mod:`paper_2509_19729_amd.binding` marshals arguments
to it.  Importing this package loads nothing; the binding loads the built
library on first use and raises if it is missing (there is no CPU fallback).
"""
__all__ = ["binding", "workloads", "build"]
