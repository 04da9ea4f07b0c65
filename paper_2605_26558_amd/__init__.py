"""MI355X-native hot path of Cassandra self-speculative decoding (HIP kernels behind a C ABI).

`binding` mirrors include/cassandra.h; importing it does not load the library until a call
is made, and a missing library is an error (there is no CPU fallback)."""
from . import binding  # noqa: F401
