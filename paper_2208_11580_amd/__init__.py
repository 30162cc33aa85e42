"""MI355X-native ExactOBS / OBQ layer solver (arxiv 2208.11580): libobc.so + its ctypes binding."""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    Context, ObcError, load_library, LIB_PATH, EXPORTS,
    STRATEGY_AUTO, STRATEGY_RANK1, STRATEGY_BLOCKED,
    OBC_OK, OBC_ERR_BAD_ARG, OBC_ERR_BAD_SHAPE, OBC_ERR_NOT_SPD, OBC_ERR_WORKSPACE,
    OBC_ERR_NUMERIC, OBC_ERR_HIP,
)
