"""Paged-KV decode attention with asynchronous KV-block prefetch for AMD MI355X (gfx950)."""
