"""MI355X-native hot path of elastic sequence parallelism (LoongServe, arXiv 2404.09526):
one GPU's share of sequence-parallel attention behind a C-ABI library."""
