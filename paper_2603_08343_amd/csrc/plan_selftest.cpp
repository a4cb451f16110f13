// Host-side self-test of the transform schedule (wht_plan.h), compiled with the host compiler only.
// For every (log2 d, log2 values-per-thread, log2 vector) the library instantiates it checks that
//   - every butterfly stage runs exactly once and only on register-resident bits,
//   - in every phase (thread, register) -> element is a bijection onto [0, d),
//   - the LDS address map is injective, 16-byte-group preserving and inside the token's region,
//   - the first and last phases give each lane whole 16-byte vectors, contiguous across lanes,
// and it emulates the whole schedule on the CPU (registers + an LDS array, phase by phase, forward
// and reverse order) against a direct +-1 sum on small sizes.
// Prints one line per configuration; exit status 0 iff all pass.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "wht_plan.h"

using namespace wht;

static unsigned thread_elem(const PhaseDesc& p, int n, int e, unsigned t) {
    unsigned off = 0;
    for (int k = 0; k < n - e; ++k) off |= ((t >> k) & 1u) << p.tb[k];
    return off;
}

static bool check(int n, int e, int v) {
    const PlanDesc pl = make_plan(n, e, v);
    const unsigned D = 1u << n, E = 1u << e, T = 1u << (n - e);
    bool ok = plan_is_complete(pl);
    const unsigned words = (lds_phys(D - 1) + 1 + 3) & ~3u;
    // address map
    std::vector<char> used(words, 0);
    for (unsigned i = 0; i < D; ++i) {
        unsigned a = lds_phys(i);
        if (a >= words || used[a]) ok = false; else used[a] = 1;
        if ((i & 3u) == 0 && ((a & 3u) != 0 || lds_phys(i + 3) != a + 3)) ok = false;
    }
    for (int p = 0; p < pl.nphase; ++p) {
        std::vector<char> seen(D, 0);
        for (unsigned t = 0; t < T; ++t)
            for (unsigned r = 0; r < E; ++r) {
                unsigned a = thread_elem(pl.ph[p], n, e, t), b = reg_elem_offset(pl.ph[p], e, (int)r);
                if (a & b) ok = false;
                unsigned el = a | b;
                if (el >= D || seen[el]) ok = false; else seen[el] = 1;
                if (lds_phys(el) != lds_phys(a) + lds_phys(b)) ok = false;
            }
    }
    // global layouts: vector bits in the low register bits, low thread bits follow on
    for (int p : {0, pl.nphase - 1}) {
        for (int q = 0; q < v; ++q) if (pl.ph[p].rb[q] != q) ok = false;
        int run = 0;
        while (run < n - e && pl.ph[p].tb[run] == v + run) ++run;
        if (n - e > 0 && run < ((n - e) < 3 ? (n - e) : 3)) ok = false;   // >= 128 contiguous bytes
    }
    // emulate on the CPU for small d
    if (n <= 11) {
        for (int reverse = 0; reverse < 2; ++reverse) {
            std::vector<double> x(D), lds(words, NAN), want(D);
            for (unsigned i = 0; i < D; ++i) x[i] = std::sin(0.37 * i + 1.0) + (i % 7) * 0.25;
            for (unsigned j = 0; j < D; ++j) {
                double s = 0;
                for (unsigned k = 0; k < D; ++k) s += (__builtin_popcount(j & k) & 1) ? -x[k] : x[k];
                want[j] = s;
            }
            std::vector<std::vector<double>> reg(T, std::vector<double>(E));
            for (int s = 0; s < pl.nphase; ++s) {
                const int p = reverse ? pl.nphase - 1 - s : s;
                const PhaseDesc& ph = pl.ph[p];
                for (unsigned t = 0; t < T; ++t) {
                    const unsigned base = thread_elem(ph, n, e, t);
                    for (unsigned r = 0; r < E; ++r) {
                        const unsigned el = base | reg_elem_offset(ph, e, (int)r);
                        reg[t][r] = (s == 0) ? x[el] : lds[lds_phys(el)];
                    }
                    for (int q = 0; q < e; ++q) {
                        if (!((ph.stages >> ph.rb[q]) & 1u)) continue;
                        for (unsigned r = 0; r < E; ++r)
                            if (!((r >> q) & 1u)) {
                                double a = reg[t][r], b = reg[t][r | (1u << q)];
                                reg[t][r] = a + b; reg[t][r | (1u << q)] = a - b;
                            }
                    }
                }
                // write-back happens after every thread has read (the barrier in the kernel)
                for (unsigned t = 0; t < T; ++t) {
                    const unsigned base = thread_elem(ph, n, e, t);
                    for (unsigned r = 0; r < E; ++r)
                        lds[lds_phys(base | reg_elem_offset(ph, e, (int)r))] = reg[t][r];
                }
            }
            double worst = 0, big = 0;
            for (unsigned j = 0; j < D; ++j) {
                worst = std::fmax(worst, std::fabs(lds[lds_phys(j)] - want[j]));
                big = std::fmax(big, std::fabs(want[j]));
            }
            if (!(worst <= 1e-9 * big)) ok = false;
        }
    }
    std::printf("n=%2d e=%d v=%d phases=%d lds_words=%u %s\n", n, e, v, pl.nphase, words, ok ? "ok" : "FAIL");
    for (int p = 0; p < pl.nphase && !ok; ++p) {
        std::printf("   phase %d regs:", p);
        for (int q = 0; q < e; ++q) std::printf(" %d", pl.ph[p].rb[q]);
        std::printf("  stages mask 0x%x\n", pl.ph[p].stages);
    }
    return ok;
}

int main(int argc, char** argv) {
    bool ok = true;
    const bool verbose = argc > 1;
    for (int v : {2, 3})
        for (int n = 5; n <= 14; ++n) {
            ok = check(n, log_e_for(n, v), v) && ok;
            if (verbose) {
                const PlanDesc pl = make_plan(n, log_e_for(n, v), v);
                for (int p = 0; p < pl.nphase; ++p) {
                    std::printf("   phase %d regs:", p);
                    for (int q = 0; q < pl.e; ++q) std::printf(" %d", pl.ph[p].rb[q]);
                    std::printf("  stages 0x%x  threads:", pl.ph[p].stages);
                    for (int k = 0; k < n - pl.e; ++k) std::printf(" %d", pl.ph[p].tb[k]);
                    std::printf("\n");
                }
            }
        }
    return ok ? 0 : 1;
}
