"""CPU oracle of the OPTIM-phase cost model and the n_persist chooser.

TEST INFRASTRUCTURE ONLY.  Plain Python, written from the paper's formulas: an iteration costs
T_FWD + max{T_BWD + T_GPU_OPTIM, T_CPU_OPTIM} with update times proportional to the parameter
size (Appendix A.1, Eq. 2 and the paragraph after Eq. 7), model states take
M_persist * n_persist + M_buffer * n_buffer (Appendix A.2, last equation), and the configuration
is found by exhaustive search under the memory capacity (Automatic Memory Management).  Here:
the optimizer phase only, 16 bytes per element per resident chunk or chunk buffer.
"""
STREAM, HOST = 0, 1


def predict(rates: dict, S: int, C: int, n_persist: int, mode: int):
    res, rest = S * n_persist, S * (C - n_persist)
    t_gpu = max(0.0, rates["gpu_s_fixed"] + rates["gpu_s_per_elem"] * res) if res else 0.0
    if mode == STREAM:
        t_other = max(0.0, rates["link_s_fixed"] + rates["link_s_per_elem"] * rest) if rest else 0.0
    else:
        t_other = max(0.0, rates["host_s_fixed"] + rates["host_s_per_elem"] * rest) if rest else 0.0
    t = max(t_gpu, t_other)
    if mode == STREAM and res and rest:
        t += rates["stream_contention"] * min(t_gpu, t_other)
    return t_gpu, t_other, t


def choose(rates: dict, S: int, C: int, budget: int, mode: int, n_slots: int):
    best = None
    for n in range(C + 1):
        buffers = n_slots if (mode == STREAM and n < C) else 0
        need = 16 * S * (n + buffers)
        if need > budget:
            continue
        t = predict(rates, S, C, n, mode)[2]
        if best is None or t < best[1]:
            best = (n, t, need, buffers)
    return best
