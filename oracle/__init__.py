"""fp64 CPU oracle for Flora's hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``flora_oracle.c`` (plain C loops) plus the two
algorithm drivers (Algorithm 1: compressed gradient accumulation; Algorithm 2:
compressed momentum with resampling) written out step by step in numpy.

Nothing in the GPU library imports this package and this package imports
nothing of the GPU library.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "flora_oracle.c"
_LIB = _HERE / "libflora_oracle.so"


def build(force: bool = False) -> Path:
    """Compile the oracle with the host C compiler (no HIP, no GPU code)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-Wall", "-Wextra", str(_SRC), "-lm", "-o", str(tmp)]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None
_c_dp = ctypes.POINTER(ctypes.c_double)
_c_u32p = ctypes.POINTER(ctypes.c_uint32)
_i64 = ctypes.c_int64
_u64 = ctypes.c_uint64
_f64 = ctypes.c_double


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(str(build()))
        L.fo_philox4x32_10.argtypes = [_c_u32p, _c_u32p, _c_u32p]
        L.fo_philox4x32_10.restype = None
        L.fo_raw_words.argtypes = [_u64, _i64, _i64, _c_u32p]
        L.fo_raw_words.restype = None
        L.fo_uniform.argtypes = [ctypes.c_uint32]
        L.fo_uniform.restype = _f64
        L.fo_A_elem.argtypes = [_u64, _i64, _i64, _i64]
        L.fo_A_elem.restype = _f64
        L.fo_materialise_A.argtypes = [_u64, _i64, _i64, _c_dp]
        L.fo_materialise_A.restype = None
        L.fo_derive_seed.argtypes = [_u64, _u64, _u64]
        L.fo_derive_seed.restype = _u64
        L.fo_compress.argtypes = [_c_dp, _i64, _i64, _i64, _u64, _f64, _f64, _c_dp]
        L.fo_compress.restype = ctypes.c_int
        L.fo_compress_regen.argtypes = [_c_dp, _i64, _i64, _i64, _u64, _f64, _f64, _c_dp]
        L.fo_compress_regen.restype = None
        L.fo_decompress.argtypes = [_c_dp, _i64, _i64, _i64, _u64, _f64, _c_dp]
        L.fo_decompress.restype = ctypes.c_int
        L.fo_decompress_regen.argtypes = [_c_dp, _i64, _i64, _i64, _u64, _f64, _c_dp]
        L.fo_decompress_regen.restype = None
        L.fo_transfer_literal.argtypes = [_c_dp, _i64, _i64, _i64, _u64, _u64, _c_dp]
        L.fo_transfer_literal.restype = ctypes.c_int
        L.fo_transfer.argtypes = [_c_dp, _i64, _i64, _i64, _u64, _u64, _c_dp, _c_dp]
        L.fo_transfer.restype = ctypes.c_int
        L.fo_sgd.argtypes = [_c_dp, _c_dp, _i64, _i64, _f64]
        L.fo_sgd.restype = None
        L.fo_factored_update.argtypes = [_c_dp, _c_dp, _i64, _i64, _c_dp, _c_dp,
                                         _f64, _f64, _f64, _f64]
        L.fo_factored_update.restype = ctypes.c_int
        L.fo_adafactor_schedule.argtypes = [_i64, _c_dp, _c_dp]
        L.fo_adafactor_schedule.restype = None
        L.fo_rms.argtypes = [_c_dp, _i64]
        L.fo_rms.restype = _f64
        L.fo_adafactor_step.argtypes = [_c_dp, _c_dp, _i64, _i64, _c_dp, _c_dp, _c_dp, ctypes.c_int,
                                        _f64, _f64, _f64, _f64, _f64, ctypes.c_int]
        L.fo_adafactor_step.restype = ctypes.c_int
        _lib = L
    return _lib


def _d(a):
    return a.ctypes.data_as(_c_dp)


def _f64c(a):
    """A C-contiguous float64 copy/view (upcasting fp32 is exact)."""
    return np.ascontiguousarray(a, dtype=np.float64)


# --------------------------------------------------------------------------
# generator
# --------------------------------------------------------------------------
def philox4x32_10(ctr, key):
    c = (ctypes.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (ctypes.c_uint32 * 4)()
    lib().fo_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def raw_words(seed: int, j: int, q: int):
    o = (ctypes.c_uint32 * 4)()
    lib().fo_raw_words(seed, j, q, o)
    return [int(x) for x in o]


def raw_words_matrix(seed: int, m: int, r: int) -> np.ndarray:
    """uint32 [m, ceil(r/4), 4]: the Philox words behind every entry of A."""
    nq = (r + 3) // 4
    out = np.empty((m, nq, 4), dtype=np.uint32)
    o = (ctypes.c_uint32 * 4)()
    L = lib()
    for j in range(m):
        for q in range(nq):
            L.fo_raw_words(seed, j, q, o)
            out[j, q, :] = o[:]
    return out


def uniform(x: int) -> float:
    return lib().fo_uniform(int(x) & 0xFFFFFFFF)


def A_elem(seed: int, j: int, k: int, r: int) -> float:
    return lib().fo_A_elem(seed, j, k, r)


def materialise_A(seed: int, m: int, r: int) -> np.ndarray:
    A = np.empty((m, r), dtype=np.float64)
    lib().fo_materialise_A(seed, m, r, _d(A))
    return A


def derive_seed(global_seed: int, matrix_id: int, epoch: int) -> int:
    return int(lib().fo_derive_seed(global_seed, matrix_id, epoch))


# --------------------------------------------------------------------------
# primitives (all return new arrays; inputs are upcast exactly to fp64)
# --------------------------------------------------------------------------
def compress(G, r: int, seed: int, state=None, a: float = 1.0, b: float = 1.0,
             regen: bool = False) -> np.ndarray:
    G = _f64c(G)
    n, m = G.shape
    st = np.zeros((n, r)) if state is None else _f64c(state).copy()
    if regen:
        lib().fo_compress_regen(_d(G), n, m, r, seed, a, b, _d(st))
    else:
        if lib().fo_compress(_d(G), n, m, r, seed, a, b, _d(st)) != 0:
            raise MemoryError
    return st


def compress_mapped(G, r: int, seed: int, input_map: str, state=None, a: float = 1.0, b: float = 1.0) -> np.ndarray:
    """Compressed EMA of another statistic (closing remark of Section 2.4, "Sublinear memory momentum"): the compression line with
    phi(G) in place of G, phi elementwise; "square" gives the second moment's term G * G."""
    G = _f64c(G)
    if input_map == "identity":
        X = G
    elif input_map == "square":
        X = G * G
    else:
        raise ValueError(input_map)
    return compress(X, r, seed, state=state, a=a, b=b)


def decompress(state, m: int, seed: int, alpha: float = 1.0, regen: bool = False) -> np.ndarray:
    st = _f64c(state)
    n, r = st.shape
    out = np.empty((n, m))
    if regen:
        lib().fo_decompress_regen(_d(st), n, m, r, seed, alpha, _d(out))
    else:
        if lib().fo_decompress(_d(st), n, m, r, seed, alpha, _d(out)) != 0:
            raise MemoryError
    return out


def transfer_literal(M, m: int, seed_old: int, seed_new: int) -> np.ndarray:
    M = _f64c(M)
    n, r = M.shape
    out = np.empty((n, r))
    if lib().fo_transfer_literal(_d(M), n, m, r, seed_old, seed_new, _d(out)) != 0:
        raise MemoryError
    return out


def transfer(M, m: int, seed_old: int, seed_new: int, return_T: bool = False):
    M = _f64c(M)
    n, r = M.shape
    out = np.empty((n, r))
    T = np.empty((r, r))
    if lib().fo_transfer(_d(M), n, m, r, seed_old, seed_new, _d(out), _d(T)) != 0:
        raise MemoryError
    return (out, T) if return_T else out


def transfer_accumulate(dst, src, m: int, seed_src: int, seed_dst: int, a: float, b: float) -> np.ndarray:
    """dst <- a dst + b (src A_src^T) A_dst, taken literally: the n x m decompression of
    ``src`` (Algorithm 1, decompression line) is compressed again under the destination's
    projection with the EMA coefficients (Algorithm 2, EMA line)."""
    src = _f64c(src)
    r = src.shape[1]
    Gt = decompress(src, m, seed_src, alpha=1.0)
    return compress(Gt, r, seed_dst, state=dst, a=a, b=b)


def sgd(W, Gt, lr: float) -> np.ndarray:
    W = _f64c(W).copy()
    Gt = _f64c(Gt)
    n, m = W.shape
    lib().fo_sgd(_d(W), _d(Gt), n, m, lr)
    return W


def factored_update(W, Gt, R, K, beta2: float, eps1: float, clip_d: float, lr: float):
    """Returns (W_new, R_new, K_new)."""
    W = _f64c(W).copy()
    Gt = _f64c(Gt)
    n, m = W.shape
    R = _f64c(R).copy()
    K = _f64c(K).copy()
    if lib().fo_factored_update(_d(W), _d(Gt), n, m, _d(R), _d(K), beta2, eps1, clip_d, lr) != 0:
        raise MemoryError
    return W, R, K


def adafactor_schedule(t: int):
    """(rho_t, beta2_t) for step t = 1, 2, ..."""
    rho, beta2 = _f64(0.0), _f64(0.0)
    lib().fo_adafactor_schedule(int(t), ctypes.byref(rho), ctypes.byref(beta2))
    return rho.value, beta2.value


def rms(X) -> float:
    X = _f64c(X)
    return float(lib().fo_rms(_d(X), X.size))


def adafactor_step(W, Gt, *, R=None, K=None, V=None, beta2: float, eps1: float = 1e-30,
                   eps2: float = 1e-3, clip_d: float = 1.0, step: float,
                   scale_parameter: bool = True):
    """One Adafactor step on one matrix.  Factored when R and K are given
    (returns (W, R, K)); unfactored when V is given (returns (W, V))."""
    W = _f64c(W).copy()
    Gt = _f64c(Gt)
    n, m = W.shape
    factored = V is None
    if factored:
        R = _f64c(R).copy()
        K = _f64c(K).copy()
        Vc = np.zeros(1)
    else:
        Vc = _f64c(V).copy()
        R = np.zeros(1)
        K = np.zeros(1)
    if lib().fo_adafactor_step(_d(W), _d(Gt), n, m, _d(R), _d(K), _d(Vc), int(factored), beta2, eps1,
                               eps2, clip_d, step, int(bool(scale_parameter))) != 0:
        raise MemoryError
    return (W, R, K) if factored else (W, Vc)


# --------------------------------------------------------------------------
# drivers
# --------------------------------------------------------------------------
def algorithm1_cycle(W_list, grads_per_step, r: int, global_seed: int, epoch: int,
                     lr: float, rule: str = "sgd", factored=None):
    """One accumulation cycle of Algorithm 1 followed by the base update.

    ``grads_per_step[i][l]`` is the gradient of matrix ``l`` at micro-step
    ``i`` (tau = len(grads_per_step)).  The accumulator starts at zero, one
    seed per matrix serves all tau compressions and the reconstruction, and
    the reconstruction is scaled by 1/tau (the accumulator is an arithmetic
    mean over the cycle; the printed 1/n is read as 1/tau).
    Returns (new W list, decompressed gradients, final accumulators).
    ``factored`` = dict(R=[...], K=[...], beta2, eps1, clip_d) for rule="factored".
    """
    tau = len(grads_per_step)
    W_out, Gt_out, C_out = [], [], []
    for l, W in enumerate(W_list):
        n, m = W.shape
        seed = derive_seed(global_seed, l, epoch)
        C = np.zeros((n, r))
        for i in range(tau):
            C = compress(grads_per_step[i][l], r, seed, state=C, a=1.0, b=1.0)
        Gt = decompress(C, m, seed, alpha=1.0 / tau)
        if rule == "sgd":
            Wn = sgd(W, Gt, lr)
        elif rule == "factored":
            Wn, Rn, Kn = factored_update(W, Gt, factored["R"][l], factored["K"][l],
                                         factored["beta2"], factored["eps1"],
                                         factored["clip_d"], lr)
            factored["R"][l], factored["K"][l] = Rn, Kn
        elif rule == "adafactor":
            # the whole Adafactor step; factored = dict(R=[..], K=[..]) or dict(V=[..]) plus
            # beta2, eps1, eps2, clip_d, step, scale_parameter
            f = factored
            kw = dict(beta2=f["beta2"], eps1=f["eps1"], eps2=f["eps2"], clip_d=f["clip_d"],
                      step=f["step"], scale_parameter=f["scale_parameter"])
            if "V" in f:
                Wn, f["V"][l] = adafactor_step(W, Gt, V=f["V"][l], **kw)
            else:
                Wn, f["R"][l], f["K"][l] = adafactor_step(W, Gt, R=f["R"][l], K=f["K"][l], **kw)
        else:
            raise ValueError(rule)
        W_out.append(Wn)
        Gt_out.append(Gt)
        C_out.append(C)
    return W_out, Gt_out, C_out


class Algorithm2:
    """Algorithm 2 (compressed momentum), one matrix set, plain SGD on the yield.

    State per matrix: M (n x r), the current seed, and the resample count
    (epoch).  At every step with t = 0 (mod kappa) -- t = 0 included, as
    printed -- a new seed is drawn, M is moved to the new projection
    (M <- M A_old^T A_new) and the step's gradient is compressed with the NEW
    projection; the yield M_{t+1} A'^T also uses the new projection.
    """

    def __init__(self, shapes, r: int, beta: float, kappa: int, global_seed: int):
        self.r, self.beta, self.kappa, self.g = r, beta, kappa, global_seed
        self.t = 0
        self.M = [np.zeros((n, r)) for (n, m) in shapes]
        self.m = [m for (n, m) in shapes]
        self.epoch = [0 for _ in shapes]
        self.seed = [derive_seed(global_seed, l, 0) for l in range(len(shapes))]
        self.transfers = 0
        self.seed_log = []

    def step(self, grads, W_list=None, lr: float = 0.0):
        """Returns (yield list, updated W list or None)."""
        ys, Ws = [], []
        resample = (self.t % self.kappa == 0)
        for l, G in enumerate(grads):
            if resample:
                self.epoch[l] += 1
                new_seed = derive_seed(self.g, l, self.epoch[l])
                Mp = transfer(self.M[l], self.m[l], self.seed[l], new_seed)
                self.seed[l] = new_seed
                self.transfers += 1
            else:
                Mp = self.M[l]
            self.M[l] = compress(G, self.r, self.seed[l], state=Mp,
                                 a=self.beta, b=1.0 - self.beta)
            y = decompress(self.M[l], self.m[l], self.seed[l], alpha=1.0)
            ys.append(y)
            if W_list is not None:
                Ws.append(sgd(W_list[l], y, lr))
        self.seed_log.append(list(self.seed))
        self.t += 1
        return ys, (Ws if W_list is not None else None)
