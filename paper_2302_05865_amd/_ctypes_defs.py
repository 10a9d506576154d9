"""ctypes mirrors of the structs in include/fa.h (layout only, no logic)."""
import ctypes

FA_P_MAX = 64
FA_ITERS_MAX = 256

(FA_OK, FA_ERR_ARG, FA_ERR_ALLOC, FA_ERR_DEVICE, FA_ERR_NONFINITE, FA_ERR_ZERO_INPUT,
 FA_ERR_TOO_LARGE) = range(7)
FA_F32, FA_BF16 = 0, 1
FA_WORKER_MAJOR, FA_ROW_MAJOR = 0, 1
FA_SOLVER_AUTO, FA_SOLVER_JACOBI16, FA_SOLVER_JACOBI = 0, 1, 2
FA_GRAM_AUTO, FA_GRAM_FP64, FA_GRAM_BF16_MATRIX = 0, 1, 2
FA_GRAM_AUTO_MIN_ROWS = 1 << 20


class FaConfig(ctypes.Structure):
    _fields_ = [("n_max", ctypes.c_int64), ("p_max", ctypes.c_int), ("dtype", ctypes.c_int),
                ("stream", ctypes.c_void_p), ("clamp_delta", ctypes.c_double),
                ("rank_tol", ctypes.c_double), ("pair_tol", ctypes.c_double),
                ("exponent_a", ctypes.c_double), ("layout", ctypes.c_int),
                ("solver", ctypes.c_int), ("wide_spin_budget", ctypes.c_int),
                ("gram", ctypes.c_int)]


class FaInfo(ctypes.Structure):
    _fields_ = [("status", ctypes.c_int), ("p", ctypes.c_int), ("m", ctypes.c_int),
                ("rank", ctypes.c_int), ("iters_done", ctypes.c_int), ("sweeps", ctypes.c_int),
                ("eigengap", ctypes.c_double),
                ("objective", ctypes.c_double * FA_ITERS_MAX),
                ("s", ctypes.c_double * FA_P_MAX), ("v", ctypes.c_double * FA_P_MAX),
                ("w", ctypes.c_double * FA_P_MAX), ("c", ctypes.c_double * FA_P_MAX),
                ("A", ctypes.c_double * (FA_P_MAX * FA_P_MAX)),
                ("K", ctypes.c_double * (FA_P_MAX * FA_P_MAX))]
