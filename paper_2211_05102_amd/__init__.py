"""MI355X-native int8-weight multiquery decode step (libpalmdecode.so + ctypes binding)."""
from .binding import Decoder, ModelDesc, PdError, lib, make_desc  # noqa: F401
