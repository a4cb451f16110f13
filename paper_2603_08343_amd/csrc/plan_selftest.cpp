// Host-side self-test of the transform schedules (wht_plan.h), compiled with the host compiler only.
// For every (schedule, log2 d) the library instantiates it checks that
//   - every stage runs exactly once (matrix-core bits included) and only on register-resident bits,
//   - in every phase (thread, register) -> element is a bijection onto [0, d),
//   - the LDS address map is injective, keeps 16-byte groups together, is additive over disjoint
//     bit sets and stays inside the token's region,
//   - the first and last phases give each lane whole 16-byte vectors, contiguous across >= 8 lanes,
//   - for the matrix-core schedule, the first layout is the MFMA operand layout the kernels assume
//     (registers = bits 0,1,2,9,tile bits; lanes = bits 3..8),
// and it emulates the whole schedule on the CPU (registers + an LDS array, phase by phase, in forward
// and in reverse order, the matrix-core rounds as butterflies on their bits) against a direct +-1
// sum on small sizes.
// Prints one line per configuration; exit status 0 iff all pass.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "wht_plan.h"

using namespace wht;

typedef unsigned (*PhysFn)(unsigned);
static unsigned phys_pad2(unsigned i) { return lds_phys_pad(i, 2); }
static unsigned phys_pad3(unsigned i) { return lds_phys_pad(i, 3); }
static unsigned phys_rot(unsigned i) { return lds_phys_rot(i); }

static unsigned thread_elem(const PhaseDesc& p, int n, int e, unsigned t) {
    unsigned off = 0;
    for (int k = 0; k < n - e; ++k) off |= ((t >> k) & 1u) << p.tb[k];
    return off;
}

static void butterfly_bits(std::vector<double>& a, unsigned bits) {
    const unsigned D = (unsigned)a.size();
    for (unsigned b = 0; (1u << b) < D; ++b) {
        if (!((bits >> b) & 1u)) continue;
        for (unsigned i = 0; i < D; ++i)
            if (!((i >> b) & 1u)) {
                const double u = a[i], w = a[i | (1u << b)];
                a[i] = u + w; a[i | (1u << b)] = u - w;
            }
    }
}

static bool check(const char* kind, const PlanDesc& pl, PhysFn phys, unsigned words, bool verbose) {
    const int n = pl.n, e = pl.e, v = pl.v;
    const unsigned D = 1u << n, E = 1u << e, T = 1u << (n - e);
    bool ok = plan_is_complete(pl);
    // address map
    std::vector<char> used(words, 0);
    for (unsigned i = 0; i < D; ++i) {
        const unsigned a = phys(i);
        if (a >= words || used[a]) ok = false; else used[a] = 1;
        if ((i & 3u) == 0 && ((a & 3u) != 0 || phys(i + 3) != a + 3)) ok = false;
    }
    for (int p = 0; p < pl.nphase; ++p) {
        std::vector<char> seen(D, 0);
        for (unsigned t = 0; t < T; ++t)
            for (unsigned r = 0; r < E; ++r) {
                const unsigned a = thread_elem(pl.ph[p], n, e, t), b = reg_elem_offset(pl.ph[p], e, (int)r);
                if (a & b) ok = false;
                const unsigned el = a | b;
                if (el >= D || seen[el]) ok = false; else seen[el] = 1;
                if (phys(el) != phys(a) + phys(b)) ok = false;
            }
    }
    // global layouts: vector bits in the low register bits, low thread bits follow on
    for (int p : {0, pl.nphase - 1}) {
        for (int q = 0; q < v; ++q) if (pl.ph[p].rb[q] != q) ok = false;
        int run = 0;
        while (run < n - e && pl.ph[p].tb[run] == v + run) ++run;
        if (n - e > 0 && run < ((n - e) < 3 ? (n - e) : 3)) ok = false;   // >= 128 contiguous bytes
    }
    if (pl.mfma_bits) {
        // operand layout of the matrix-core rounds
        const PhaseDesc& f = pl.ph[0];
        if (pl.mfma_bits != 0x3ffu || v != 3) ok = false;
        if (f.rb[0] != 0 || f.rb[1] != 1 || f.rb[2] != 2 || f.rb[3] != 9) ok = false;
        for (int q = 4; q < e; ++q) if (f.rb[q] != 10 + (q - 4)) ok = false;
        for (int k = 0; k < 6; ++k) if (f.tb[k] != 3 + k) ok = false;
        // every layout keeps lanes on bits 3..8, so the exchange is between waves only
        for (int p = 0; p < pl.nphase; ++p)
            for (int k = 0; k < 6; ++k) if (pl.ph[p].tb[k] != 3 + k) ok = false;
    }
    // emulate on the CPU for small d
    if (n <= 12) {
        for (int reverse = 0; reverse < 2; ++reverse) {
            std::vector<double> x(D), lds(words, NAN), want(D);
            for (unsigned i = 0; i < D; ++i) x[i] = std::sin(0.37 * i + 1.0) + (i % 7) * 0.25;
            want = x;
            butterfly_bits(want, D - 1);
            if (n <= 9) {       // and the direct sum itself on the smallest sizes
                for (unsigned j = 0; j < D; ++j) {
                    double s = 0;
                    for (unsigned k = 0; k < D; ++k) s += (__builtin_popcount(j & k) & 1) ? -x[k] : x[k];
                    if (std::fabs(s - want[j]) > 1e-9 * (1 + std::fabs(s))) ok = false;
                }
            }
            // the matrix-core rounds come first going forward (on the data as loaded) ...
            if (!reverse) butterfly_bits(x, pl.mfma_bits);
            std::vector<std::vector<double>> reg(T, std::vector<double>(E));
            for (int s = 0; s < pl.nphase; ++s) {
                const int p = reverse ? pl.nphase - 1 - s : s;
                const PhaseDesc& ph = pl.ph[p];
                for (unsigned t = 0; t < T; ++t) {
                    const unsigned base = thread_elem(ph, n, e, t);
                    for (unsigned r = 0; r < E; ++r) {
                        const unsigned el = base | reg_elem_offset(ph, e, (int)r);
                        reg[t][r] = (s == 0) ? x[el] : lds[phys(el)];
                    }
                    for (int q = 0; q < e; ++q) {
                        if (!((ph.stages >> ph.rb[q]) & 1u)) continue;
                        for (unsigned r = 0; r < E; ++r)
                            if (!((r >> q) & 1u)) {
                                const double a = reg[t][r], b = reg[t][r | (1u << q)];
                                reg[t][r] = a + b; reg[t][r | (1u << q)] = a - b;
                            }
                    }
                }
                // write-back happens after every thread has read (the barrier in the kernel)
                for (unsigned t = 0; t < T; ++t) {
                    const unsigned base = thread_elem(ph, n, e, t);
                    for (unsigned r = 0; r < E; ++r)
                        lds[phys(base | reg_elem_offset(ph, e, (int)r))] = reg[t][r];
                }
            }
            std::vector<double> got(D);
            for (unsigned j = 0; j < D; ++j) got[j] = lds[phys(j)];
            // ... and last in reverse (on the registers of the first layout)
            if (reverse) butterfly_bits(got, pl.mfma_bits);
            double worst = 0, big = 0;
            for (unsigned j = 0; j < D; ++j) {
                worst = std::fmax(worst, std::fabs(got[j] - want[j]));
                big = std::fmax(big, std::fabs(want[j]));
            }
            if (!(worst <= 1e-9 * big)) ok = false;
        }
    }
    std::printf("%-9s n=%2d e=%d v=%d phases=%d lds_words=%u %s\n", kind, n, e, v, pl.nphase, words,
                ok ? "ok" : "FAIL");
    if (verbose || !ok)
        for (int p = 0; p < pl.nphase; ++p) {
            std::printf("   phase %d regs:", p);
            for (int q = 0; q < e; ++q) std::printf(" %d", pl.ph[p].rb[q]);
            std::printf("  stages 0x%x  threads:", pl.ph[p].stages);
            for (int k = 0; k < n - e; ++k) std::printf(" %d", pl.ph[p].tb[k]);
            std::printf("\n");
        }
    return ok;
}

// Rows of 12 * 2^m elements on 16 * 2^m slots: the slot map must be a bijection from the valid slots
// onto the row, additive over bits, and "Sylvester butterflies on every slot bit but 4..7, the
// order-12 round matrix along bits 3..7" must equal the definition
//     out[j] = sum_k P12[j / L][k / L] * (-1)^popcount(j & k & (L - 1)) * x[k],   L = 2^m.
static bool check_twelve(int n) {
    const unsigned S = 1u << n, L = S / 16, D = 12 * L;
    bool ok = true;
    std::vector<int> hit(D, 0);
    for (unsigned s = 0; s < S; ++s) {
        if (!twelve_valid(s)) continue;
        const unsigned el = twelve_elem(s, n);
        if (el >= D) { ok = false; continue; }
        ++hit[el];
        for (int b = 0; b < n; ++b)        // additivity over single bits
            if ((s >> b) & 1u)
                if (twelve_elem(s, n) != twelve_elem(s & ~(1u << b), n) + twelve_elem(1u << b, n)) ok = false;
        if ((s & 7u) == 0 && twelve_elem(s | 7u, n) != el + 7) ok = false;    // 8-element vectors stay whole
    }
    for (unsigned el = 0; el < D; ++el) if (hit[el] != 1) ok = false;
    // the definition, on a small pseudo-random integer row (exact in double)
    std::vector<double> x(D), want(D), slot(S, 0.0);
    uint32_t rng = 12345u + (uint32_t)n;
    for (unsigned k = 0; k < D; ++k) { rng = rng * 1664525u + 1013904223u; x[k] = (double)((int)(rng >> 24) - 128); }
    if (n <= 12) {
        for (unsigned j = 0; j < D; ++j) {
            double acc = 0;
            for (unsigned k = 0; k < D; ++k) {
                const int p = ((paley12_minus_row(j / L) >> (k / L)) & 1u) ? -1 : 1;
                const int sy = (__builtin_popcount(j & k & (L - 1)) & 1) ? -1 : 1;
                acc += p * sy * x[k];
            }
            want[j] = acc;
        }
        for (unsigned s = 0; s < S; ++s) if (twelve_valid(s)) slot[s] = x[twelve_elem(s, n)];
        for (int b = 0; b < n; ++b) {                       // Sylvester bits: all but 3..7
            if (b >= 3 && b <= 7) continue;
            for (unsigned s = 0; s < S; ++s)
                if (!((s >> b) & 1u)) {
                    const double a = slot[s], c = slot[s | (1u << b)];
                    slot[s] = a + c; slot[s | (1u << b)] = a - c;
                }
        }
        std::vector<double> out(S, 0.0);
        for (unsigned s = 0; s < S; ++s) {                  // the 32 x 32 round along bits 3..7
            const unsigned m_out = (s >> 3) & 31u, rest = s & ~(31u << 3);
            double acc = 0;
            for (unsigned m_in = 0; m_in < 32; ++m_in)
                acc += twelve_round_entry(m_in, m_out) * slot[rest | (m_in << 3)];
            out[s] = acc;
        }
        for (unsigned s = 0; s < S; ++s) {
            if (twelve_valid(s)) { if (out[s] != want[twelve_elem(s, n)]) ok = false; }
            else if (out[s] != 0.0) ok = false;             // padding stays zero
        }
    }
    std::printf("twelve    n=%2d row=%u slots=%u %s\n", n, D, S, ok ? "ok" : "FAIL");
    return ok;
}

int main(int argc, char** argv) {
    if (argc > 1 && std::string(argv[1]) == "--p12") {     // print the order-12 factor, rows of +/-
        for (unsigned r = 0; r < 12; ++r) {
            for (unsigned c = 0; c < 12; ++c) std::putchar(((paley12_minus_row(r) >> c) & 1u) ? '-' : '+');
            std::putchar('\n');
        }
        return 0;
    }
    bool ok = true;
    const bool verbose = argc > 1;
    for (int n = 10; n <= 14; ++n) ok = check_twelve(n) && ok;
    for (int v : {2, 3})
        for (int n = 5; n <= (v == 2 ? 13 : 14); ++n) {
            const PlanDesc pl = make_plan(n, log_e_for(n, v), v);
            ok = check("butterfly", pl, v == 2 ? phys_pad2 : phys_pad3, lds_words_pad(1u << n, v), verbose) && ok;
        }
    for (int n = 10; n <= 14; ++n)
        for (int backward = 0; backward < 2; ++backward) {
            if (backward && mfma_log_tiles(n, true) == mfma_log_tiles(n, false)) continue;
            const PlanDesc pl = make_mfma_plan(n, mfma_log_tiles(n, backward != 0));
            ok = check("mfma", pl, phys_rot, 1u << n, verbose) && ok;
        }
    return ok ? 0 : 1;
}
