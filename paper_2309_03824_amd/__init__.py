"""MI355X (gfx950) library for low-rank-decomposed layers: SVD pairs and Tucker-2 convolutions with
rank quantization and sequential freezing.  `binding` mirrors include/lrd.h; `factorize` is the
one-time host-side decomposition that produces the factors the kernels consume."""
from . import binding  # noqa: F401  (fails loudly if liblrd.so cannot be loaded)
from . import factorize  # noqa: F401
