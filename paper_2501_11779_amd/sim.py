"""ctypes front end of the pipeline simulator in libgh_tier2.so (include/gh_sim.h); no torch."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgh_tier2.so")
SIM_EXPORTS = ("gh_sim_two_tier", "gh_sim_single_tier", "gh_sim_tbt", "gh_sim_if_pp", "gh_sim_if_gh",
               "gh_sim_if_tp", "gh_sim_max_batch")

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first")
        L = C.CDLL(LIB_PATH)
        D, I = C.c_double, C.c_int32
        DP = C.POINTER(C.c_double)
        L.gh_sim_two_tier.restype = I
        L.gh_sim_two_tier.argtypes = [I, I, I, I, D, D, D, D, D, I, DP]
        L.gh_sim_single_tier.restype = I
        L.gh_sim_single_tier.argtypes = [I, I, I, I, D, D, D, I, DP]
        L.gh_sim_tbt.restype = D
        L.gh_sim_tbt.argtypes = [DP, I, I]
        L.gh_sim_if_pp.restype = I
        L.gh_sim_if_pp.argtypes = [I, I, D, D]
        L.gh_sim_if_gh.restype = I
        L.gh_sim_if_gh.argtypes = [D, D, D]
        L.gh_sim_if_tp.restype = I
        L.gh_sim_if_tp.argtypes = [I, D, D]
        L.gh_sim_max_batch.restype = C.c_int64
        L.gh_sim_max_batch.argtypes = [D, D, I]
        _lib = L
    return _lib


def gh_sim_two_tier(N, K, IF, E, t_net_12, t_net_21, t_net_rtt, t_c_att, t_c_nonatt, later_first=True):
    out = (C.c_double * max(E, 1))()
    st = lib().gh_sim_two_tier(N, K, IF, E, t_net_12, t_net_21, t_net_rtt, t_c_att, t_c_nonatt,
                               int(later_first), out)
    if st != 0:
        raise ValueError(f"gh_sim_two_tier: status {st}")
    return list(out)[:E]


def gh_sim_single_tier(N, K, IF, E, t_net_link, t_net_rtt, t_c, later_first=True):
    out = (C.c_double * max(E, 1))()
    st = lib().gh_sim_single_tier(N, K, IF, E, t_net_link, t_net_rtt, t_c, int(later_first), out)
    if st != 0:
        raise ValueError(f"gh_sim_single_tier: status {st}")
    return list(out)[:E]


def gh_sim_tbt(gen_ts, warmup=2):
    arr = (C.c_double * len(gen_ts))(*gen_ts)
    return lib().gh_sim_tbt(arr, len(gen_ts), warmup)


def gh_sim_if_pp(K, N, t_n, t_c):
    return lib().gh_sim_if_pp(K, N, t_n, t_c)


def gh_sim_if_gh(t_c2_att, t_n, t_c1_noatt):
    return lib().gh_sim_if_gh(t_c2_att, t_n, t_c1_noatt)


def gh_sim_if_tp(K, t_n, t_c_min):
    return lib().gh_sim_if_tp(K, t_n, t_c_min)


def gh_sim_max_batch(C_max, M, n_in_flight):
    return lib().gh_sim_max_batch(C_max, M, n_in_flight)
