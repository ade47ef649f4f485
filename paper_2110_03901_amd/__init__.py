"""Implicit channel-first im2col convolution for AMD MI355X (gfx950).

The product is the HIP library behind include/iconv.h; `binding` is its thin ctypes wrapper.
Importing `binding` fails loudly if the library has not been built."""
