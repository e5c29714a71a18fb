"""MuSe (Multipole Semantic Attention) hot path for MI355X: thin Python binding over libmuse.so."""
