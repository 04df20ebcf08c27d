"""MI355X-native masked convolution (semi-structured activation sparsity) -- Python face.

`binding` mirrors the C ABI of libsparse_conv.so one to one; `runtime` adds the tensor
marshalling helpers and the small layer/network drivers the tests and the benchmark use.
"""
from . import binding  # noqa: F401
