"""CPU oracle: test infrastructure only.  Never imported by the product package."""
from .binding import Oracle, ops, conv_out_size, set_threads  # noqa: F401
