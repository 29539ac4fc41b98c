"""MI355X-native partially-linear FFN (folded product + online predictor + exact
fallback).  Importing the package does not load the GPU library; that happens on
first use of :mod:`paper_2501_10054_amd.tardis`."""

__all__ = ["synth"]
