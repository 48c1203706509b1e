"""MI355X-native error-bounded compression of fp32 activation tensors.

The hot path (pre-quantisation, 2D Lorenzo, outlier split, histogram, canonical
Huffman, chunked bit-packing and the inverse) runs entirely in hand-written HIP
kernels behind the C ABI declared in ``include/cmpz.h``; :mod:`.binding` is the
argument-marshalling layer over it.  Importing this package does not load the
library; the first use of :mod:`.binding` does, and fails loudly if it is absent.
"""
