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
    """(t_gpu, t_other, t_step).  The resident part and the other part run side by side and the longer one
    decides (the paper's max), except that the other part cannot start before the gradient norm is final:
    the share `gpu_serial_share` of the resident part (the gradient pack and its reduction, which come
    before the norm) is served first, the rest of the resident part runs beside the other part.  With
    global-norm clipping no update - on the GPU, through the chunk buffers or on the host - may read a
    gradient before that.  (Reading: the paper overlaps its CPU update with the backward pass and has no
    clipping; share 0 gives its plain max.)"""
    res, rest = S * n_persist, S * (C - n_persist)
    t_gpu = max(0.0, rates["gpu_s_fixed"] + rates["gpu_s_per_elem"] * res) if res else 0.0
    if mode == STREAM:
        t_other = max(0.0, rates["link_s_fixed"] + rates["link_s_per_elem"] * rest) if rest else 0.0
    else:
        t_other = max(0.0, rates["host_s_fixed"] + rates["host_s_per_elem"] * rest) if rest else 0.0
    if not rest:
        return t_gpu, t_other, t_gpu
    t_first = rates.get("gpu_serial_share", 0.0) * t_gpu
    t_beside = t_gpu - t_first
    t = t_first + max(t_beside, t_other)
    if mode == STREAM and res:
        t += rates["stream_contention"] * min(t_beside, t_other)
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
