// Hardware-aware shard widths for a class-column split (host code, no GPU).
//
// Section 3.3.1 of the paper balances a `split` TaskGraph over devices of unequal capacity by
// uneven sharding in the splitting dimension: load ratios proportional to the devices' FLOP/s
// minimise the formula given there, and Algorithm 1 ("Memory-Constraint Load Balancing") then moves
// load off devices that would run out of memory.  Here the load of device i is the width w_i of
// its shard in class columns; it uses (w_i / C) TG_mem of memory and (w_i / C) TG_flop of work.
#include <math.h>
#include <stdint.h>

#include <vector>

#include "../../include/whalesplit.h"

namespace {

struct Device {
    double flops, mem;     // DF_i, DM_i
    int32_t width;         // columns currently assigned
    int32_t cap;           // most columns that fit its memory
    bool over;             // on the out-of-memory list
    bool has_room;         // on the free list
};

double mem_util(int32_t w, int32_t C, double tg_mem, double dm) { return ((double)w / (double)C) * tg_mem / dm; }
double flop_util(int32_t w, int32_t C, double tg_flop, double df) { return ((double)w / (double)C) * tg_flop / df; }

int32_t columns_that_fit(int32_t C, double tg_mem, double dm) {
    double guess = floor(dm / tg_mem * (double)C);
    int32_t w = guess < 0.0 ? 0 : (guess > (double)C ? C : (int32_t)guess);
    while (w < C && mem_util(w + 1, C, tg_mem, dm) <= 1.0) ++w;
    while (w > 0 && mem_util(w, C, tg_mem, dm) > 1.0) --w;
    return w;
}

bool positive_finite(double v) { return isfinite(v) && v > 0.0; }

}  // namespace

extern "C" int ws_balance_widths(int32_t N, const double* DF, const double* DM, double TG_flop, double TG_mem,
                                 int32_t C, int32_t* widths, int32_t* feasible) {
    if (!DF || !DM || !widths || !feasible) return WS_ERR_NULL;
    if (N <= 0 || C <= 0) return WS_ERR_SHAPE;
    if (!positive_finite(TG_flop) || !positive_finite(TG_mem)) return WS_ERR_RANGE;
    for (int32_t i = 0; i < N; ++i)
        if (!positive_finite(DF[i]) || !positive_finite(DM[i])) return WS_ERR_RANGE;

    std::vector<Device> dev(N);
    double total = 0.0;
    for (int32_t i = 0; i < N; ++i) total += DF[i];

    // proportional shares, rounded by largest remainder (ties to the lower index)
    std::vector<double> frac(N);
    int64_t assigned = 0;
    for (int32_t i = 0; i < N; ++i) {
        const double q = DF[i] / total * (double)C;
        const double fl = floor(q);
        dev[i] = Device{DF[i], DM[i], (int32_t)fl, 0, false, false};
        frac[i] = q - fl;
        assigned += dev[i].width;
    }
    for (int64_t left = (int64_t)C - assigned; left > 0; --left) {
        int32_t best = -1;
        for (int32_t i = 0; i < N; ++i)
            if (frac[i] >= 0.0 && (best < 0 || frac[i] > frac[best])) best = i;
        dev[best].width += 1;
        frac[best] = -1.0;      // one extra column per device at most
    }

    int32_t n_over = 0, n_room = 0;
    for (int32_t i = 0; i < N; ++i) {
        dev[i].cap = columns_that_fit(C, TG_mem, dev[i].mem);
        dev[i].over = mem_util(dev[i].width, C, TG_mem, dev[i].mem) > 1.0;
        dev[i].has_room = !dev[i].over;
        n_over += dev[i].over;
        n_room += dev[i].has_room;
    }

    while (n_over > 0 && n_room > 0) {
        // peak: the over-memory device with the highest memory utilisation
        int32_t peak = -1, valley = -1;
        double peak_mu = 0.0, valley_fu = 0.0, valley_mu = 0.0;
        for (int32_t i = 0; i < N; ++i) {
            const double mu = mem_util(dev[i].width, C, TG_mem, dev[i].mem);
            if (dev[i].over && (peak < 0 || mu > peak_mu)) { peak = i; peak_mu = mu; }
            if (dev[i].has_room) {
                const double fu = flop_util(dev[i].width, C, TG_flop, dev[i].flops);
                if (valley < 0 || fu < valley_fu || (fu == valley_fu && mu < valley_mu)) {
                    valley = i; valley_fu = fu; valley_mu = mu;
                }
            }
        }
        const int32_t need = dev[peak].width - dev[peak].cap;
        const int32_t room = dev[valley].cap - dev[valley].width;
        const int32_t b = need < room ? need : room;
        if (b > 0) {
            dev[peak].width -= b;
            dev[valley].width += b;
        }
        if (dev[peak].width <= dev[peak].cap) {
            dev[peak].over = false;
            --n_over;
        } else {
            dev[valley].has_room = false;
            --n_room;
        }
    }
    for (int32_t i = 0; i < N; ++i) widths[i] = dev[i].width;
    *feasible = n_over == 0 ? 1 : 0;
    return WS_OK;
}
