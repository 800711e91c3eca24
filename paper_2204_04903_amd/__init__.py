"""MI355X-native packed multi-field embedding layer (forward, backward, sparse Adagrad).

`binding` mirrors the C ABI of include/pk.h one to one; `layer.PackedEmbedding`
only allocates torch device buffers and passes their addresses through.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, PkError, build, lib
