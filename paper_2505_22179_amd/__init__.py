"""MI355X-native W4A16 small-M linear layer and tree-verify attention (C-ABI library + binding).

`inputs` holds the seeded synthetic input generators; `binding` is the thin ctypes layer over
libw4a16.so.  Importing the package does not load the library; calling into `binding` does and
fails loudly if it has not been built."""
