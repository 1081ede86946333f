"""C-K-S conv-layer operators for MI355X (gfx950): Python binding over libcks.so."""
