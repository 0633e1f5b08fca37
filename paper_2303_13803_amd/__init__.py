"""MI355X-native core of matching-based GPU-sharing scheduling: pair scoring
and maximum-weight matching as HIP kernels behind a C ABI (libmuxmatch.so)."""
from .binding import (ERR_ARG, ERR_CERT, ERR_HIP, ERR_NOT_CONVERGED, ERR_RANGE, ERR_SHAPE,
                      INFEASIBLE, OK, Context, MuxmatchError, Predictor, Result, strerror)
