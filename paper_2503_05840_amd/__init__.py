"""MI355X-native slim-attention decode path (K-cache only MHA generation step).

`synth` draws the seeded inputs; `binding` is the thin ctypes layer over the C-ABI library
built from `csrc/` (loaded lazily, so importing the package needs neither a GPU nor the
built library)."""
