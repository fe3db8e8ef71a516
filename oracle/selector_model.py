"""Plain transcription of the paper's analytical model (TEST INFRASTRUCTURE ONLY).

Section IV of the paper: Algorithm 3 (compute latency of a shared-memory tile), Algorithm 4
(active CUs in the last timestep, number of waves), Algorithm 5 (cache hit rate of a cache
tile), Algorithm 6 (factorisations of the CU count of a cache scope), Algorithm 7 (memory
latency of one loop iteration), Algorithm 8 (latency of one output tile) and Algorithm 9
(total latency).  The `alg*` functions take the steps in the paper's order and notation,
with no reading added.  `predict` composes them for one kernel variant the way the shipped
selector is specified to (every place where the paper is silent or inconsistent is marked
READING and listed in the design doc); the tests compare the C++ selector's terms with it.

Shares no code with the product; nothing under the product package imports this module.
The selector's final pick is a heuristic ranked empirically against a sweep, so beyond the
structural pins in tests/test_selector_model.py its parity is unpinned by the paper.
"""
import math


# ---------------------------------------------------------------- the paper's algorithms

def alg3_compute_latency(mi_m, mi_n, mi_k, mt_m, mt_n, mt_k, l_mi):
    """Algorithm 3: matrix instructions per shared-memory tile and their latency."""
    n_mi_m = math.ceil(mt_m / mi_m)
    n_mi_n = math.ceil(mt_n / mi_n)
    n_mi_k = math.ceil(mt_k / mi_k)
    n_mi = n_mi_m * n_mi_n * n_mi_k
    l_mt = l_mi * n_mi
    return n_mi, l_mt


def alg4_occupancy(M, N, mt_m, mt_n, n_cu):
    """Algorithm 4 as printed: (active_cu, omega, T_out); active_cu is T_out mod N_CU."""
    n_mt_m = math.ceil(M / mt_m)
    n_mt_n = math.ceil(N / mt_n)
    t_out = n_mt_m * n_mt_n
    omega = math.ceil(t_out / n_cu)
    active_cu = t_out % n_cu
    return active_cu, omega, t_out


def alg5_hit_rate(m_t, n_t, M_T, N_T, K_T):
    """Algorithm 5: hit rate of an m_t x n_t cache tile of M_T x N_T x K_T workgroup tiles."""
    U = (m_t * M_T + n_t * N_T) * K_T          # uncached reads
    R = (m_t * n_t) * (M_T + N_T) * K_T        # total reads
    h = 1 - U / R
    return h


def alg6_factorizations(n_cu_cache):
    """Algorithm 6: every (f_m, f_n) with f_m * f_n = N_CU_cache, in ascending f_m."""
    F = []
    for i in range(1, n_cu_cache + 1):
        if n_cu_cache % i == 0:
            F.append((i, n_cu_cache // i))
    return F


def alg7_memory_latency(ld_cu, C, H1, H2, R_L1, R_1, R_2, R_MEM, L_lat):
    """Algorithm 7 as printed (any consistent unit of data per cycle)."""
    L_cu_lat = ld_cu / R_L1
    T = ld_cu * C
    L_1 = T / R_1
    T_2 = (1 - H1) * T
    L_2 = T_2 / R_2
    T_M = (1 - H2) * T_2
    L_MEM = T_M / R_MEM + L_lat
    return max(L_cu_lat, L_1, L_2, L_MEM)


def alg8_tile_latency(K, k_t, l_mem, l_compute, a, m_t, n_t, R_mem):
    """Algorithm 8 as printed."""
    l_prologue = l_mem
    l_epilogue = a * m_t * n_t / R_mem
    l_loopiter = max(l_compute, l_mem)
    I = math.ceil(K / k_t) - 1
    return l_prologue + l_epilogue + l_loopiter * I


def alg9_total_latency(M, N, m_t, n_t, n_cu, l_tile):
    """Algorithm 9 as printed."""
    n_m = math.ceil(M / m_t)
    n_n = math.ceil(N / n_t)
    n_waves = math.ceil(n_m * n_n / n_cu)
    return n_waves * l_tile
