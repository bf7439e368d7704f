"""fupr: inference of fusion-transformed, filter-pruned residual networks on
AMD gfx950.  `binding` mirrors include/fupr.h; `network` turns a pre-trained
model description into a runnable model.  Importing `binding` fails if
libfupr.so has not been built; there is no fallback implementation."""
