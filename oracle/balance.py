"""Oracle for the hardware-aware width balancer (intra-TaskGraph load balance of a `split`).

TEST INFRASTRUCTURE ONLY; shares no code with the library and never imports it.

It takes the steps of the paper's "Memory-Constraint Load Balancing" algorithm (Section 3.3.1,
Algorithm 1) in the paper's order and with its names: load ratios start proportional to the
devices' computing capacity (the unconstrained minimiser of the formula in Section 3.3.1); while
some device is over its memory and some device has room, load is shifted from the over-memory
device with the highest memory utilisation (the peak) to the device with room that has the lowest
(flop utilisation, memory utilisation) (the valley).

For a `split` TaskGraph the load is the width of a device's shard, in whole class columns
(Section 3.3.1: uneven sharding in the splitting dimension).  Readings where the paper is silent:
  * devices are numbered 0 .. N-1; the norm in the formula is the absolute value;
  * the unit of `shift_load` is one class column; device i holding w_i of C columns uses
    (w_i / C) * TG_mem of memory and (w_i / C) * TG_flop of work;
  * the initial integer widths are the proportional shares rounded by largest remainder
    (ties to the lower device index);
  * `shift_load(peak, valley)` moves b columns, b = the smaller of what the peak must shed to fit
    its memory and what the valley can take without exceeding its own; the shift is applied in
    either case and it "succeeds" when the peak then fits;
  * ties in argmax / argmin go to the lower device index.
"""
import math


def mem_util(w, C, TG_mem, DM_i):
    return (w / C) * TG_mem / DM_i


def flop_util(w, C, TG_flop, DF_i):
    return (w / C) * TG_flop / DF_i


def max_columns(C, TG_mem, DM_i):
    """Largest width whose memory utilisation on this device does not exceed 1."""
    w = int(math.floor(DM_i / TG_mem * C))
    w = max(0, min(C, w))
    while w < C and mem_util(w + 1, C, TG_mem, DM_i) <= 1.0:
        w += 1
    while w > 0 and mem_util(w, C, TG_mem, DM_i) > 1.0:
        w -= 1
    return w


def proportional_widths(C, DF):
    """Integer widths closest to C * DF_i / sum(DF): floors, then the leftover columns one each to the
    largest fractional parts."""
    total = 0.0
    for f in DF:
        total += f
    q = [DF[i] / total * C for i in range(len(DF))]
    w = [int(math.floor(x)) for x in q]
    left = C - sum(w)
    order = sorted(range(len(DF)), key=lambda i: (-(q[i] - w[i]), i))
    for i in order[:left]:
        w[i] += 1
    return w


def balance_widths(C, DF, DM, TG_flop, TG_mem):
    """Returns (widths, feasible).  Algorithm 1 with the column as the unit of load."""
    N = len(DF)
    widths = proportional_widths(C, DF)
    load_ratios = [widths[i] / C for i in range(N)]                      # kept for the reader: L_i
    mem_utils = [mem_util(widths[i], C, TG_mem, DM[i]) for i in range(N)]
    flop_utils = [flop_util(widths[i], C, TG_flop, DF[i]) for i in range(N)]
    oom_devices = [i for i in range(N) if mem_utils[i] > 1.0]
    free_devices = [i for i in range(N) if not mem_utils[i] > 1.0]

    def shift_load(peak, valley):
        need = widths[peak] - max_columns(C, TG_mem, DM[peak])
        room = max_columns(C, TG_mem, DM[valley]) - widths[valley]
        b = min(need, room)
        if b > 0:
            widths[peak] -= b
            widths[valley] += b
        return widths[peak] <= max_columns(C, TG_mem, DM[peak])

    def update_profile(i):
        load_ratios[i] = widths[i] / C
        mem_utils[i] = mem_util(widths[i], C, TG_mem, DM[i])
        flop_utils[i] = flop_util(widths[i], C, TG_flop, DF[i])

    while oom_devices and free_devices:
        peak_device = min(oom_devices, key=lambda i: (-mem_utils[i], i))
        valley_device = min(free_devices, key=lambda i: (flop_utils[i], mem_utils[i], i))
        ok = shift_load(peak_device, valley_device)
        update_profile(peak_device)
        update_profile(valley_device)
        if ok:
            oom_devices.remove(peak_device)
        else:
            free_devices.remove(valley_device)
    return widths, not oom_devices


def objective(widths, C, DF):
    """The quantity the formula of Section 3.3.1 minimises: sum_i |L_i - DF_i / sum(DF)|."""
    total = sum(DF)
    return sum(abs(widths[i] / C - DF[i] / total) for i in range(len(DF)))
