// Compile-time schedule of one token's fast Walsh-Hadamard transform across a group of threads.
//
// A token has d = 2^n elements.  It is held by 2^(n-e) threads, 2^e values per thread, in float32
// registers.  A butterfly stage on element-index bit b (paper Fig. 2: pairs whose indices differ by
// the stride 2^b) costs one add or subtract per element when bit b is a bit of the *register*
// index, so the schedule is a short list of layouts ("phases"); each phase names which e element
// bits are register-resident, the stages run on those, and between phases the token is re-dealt
// through LDS.  Stages commute (they act on different index bits), so any order gives H_raw x.
//
// The first and the last layout keep element bits 0..v-1 in registers (2^v elements = one 16-byte
// global vector) and give the lowest thread bits the next element bits, so that global loads and
// stores are 16 bytes per lane and contiguous across lanes.
#pragma once

namespace wht {

constexpr int kMaxRegBits = 6;
constexpr int kMaxBits = 16;
constexpr int kMaxPhases = 5;

struct PhaseDesc {
    int rb[kMaxRegBits];   // rb[q]: element-index bit carried by bit q of the register index
    int tb[kMaxBits];      // tb[k]: element-index bit carried by bit k of the thread index
    unsigned stages;       // element bits butterflied while the token is in this layout
};

struct PlanDesc {
    int n, e, v, nphase;
    unsigned mfma_bits;    // element bits transformed by the matrix-core rounds (in the first layout)
    PhaseDesc ph[kMaxPhases];
};

constexpr int popcount_u(unsigned m) { int c = 0; while (m) { c += m & 1u; m >>= 1; } return c; }
constexpr int lowest_bit(unsigned m) { int b = 0; while (!(m & 1u)) { m >>= 1; ++b; } return b; }

constexpr unsigned reg_mask(const PhaseDesc& p, int e) {
    unsigned m = 0;
    for (int q = 0; q < e; ++q) m |= 1u << p.rb[q];
    return m;
}

constexpr void fill_thread_bits(PhaseDesc& p, int n, int e) {
    const unsigned inreg = reg_mask(p, e);
    int k = 0;
    for (int b = 0; b < n; ++b)
        if (!((inreg >> b) & 1u)) p.tb[k++] = b;
    for (; k < kMaxBits; ++k) p.tb[k] = 0;
}

// log2(values per thread) the library uses for a given log2 d: 32 values where the token is large
// enough to keep 8 threads busy, never fewer than one 16-byte vector.
constexpr int log_e_for(int logd, int logv) {
    int e = logd - 3;
    if (e > 5) e = 5;
    if (e < logv) e = logv;
    return e;
}

// n = log2 d, e = log2(values per thread), v = log2(elements per 16-byte vector);  v <= e <= n.
constexpr PlanDesc make_plan(int n, int e, int v) {
    PlanDesc pl{};
    pl.n = n; pl.e = e; pl.v = v; pl.nphase = 0; pl.mfma_bits = 0;
    const unsigned all = (1u << n) - 1u;
    unsigned undone = all;

    // first phase: the vector bits and the top e-v bits
    PhaseDesc first{};
    for (int q = 0; q < v; ++q) first.rb[q] = q;
    for (int q = v; q < e; ++q) first.rb[q] = n - (e - v) + (q - v);
    first.stages = reg_mask(first, e);
    fill_thread_bits(first, n, e);
    undone &= ~first.stages;
    pl.ph[pl.nphase++] = first;
    if (n == e) return pl;

    // the last phase can take e-v new bits: reserve the top ones still undone for it -- but only
    // bits >= v+3, so that its three lowest thread bits stay element bits v..v+2 (eight lanes
    // cover 128 contiguous bytes of the global store)
    unsigned reserved = 0;
    {
        int taken = 0;
        for (int b = n - 1; b >= v + 3 && taken < e - v; --b)
            if ((undone >> b) & 1u) { reserved |= 1u << b; ++taken; }
    }
    // middle phases: windows of e consecutive element bits, lowest undone bit first
    unsigned middle = undone & ~reserved;
    while (middle) {
        int lo = lowest_bit(middle);
        if (lo > n - e) lo = n - e;
        PhaseDesc mid{};
        for (int q = 0; q < e; ++q) mid.rb[q] = lo + q;
        mid.stages = reg_mask(mid, e) & undone;
        fill_thread_bits(mid, n, e);
        undone &= ~mid.stages;
        middle &= ~mid.stages;
        pl.ph[pl.nphase++] = mid;
    }
    // last phase: vector bits, whatever is still undone, then top bits to fill the register index
    PhaseDesc last{};
    for (int q = 0; q < v; ++q) last.rb[q] = q;
    {
        int q = v;
        unsigned used = (1u << v) - 1u;
        for (int b = 0; b < n && q < e; ++b)
            if ((undone >> b) & 1u) { last.rb[q++] = b; used |= 1u << b; }
        for (int b = n - 1; b >= 0 && q < e; --b)
            if (!((used >> b) & 1u)) { last.rb[q++] = b; used |= 1u << b; }
        // keep the chunk bits ascending so register order follows memory order
        for (int i = v; i < e; ++i)
            for (int j = i + 1; j < e; ++j)
                if (last.rb[j] < last.rb[i]) { int t = last.rb[i]; last.rb[i] = last.rb[j]; last.rb[j] = t; }
    }
    last.stages = undone;
    fill_thread_bits(last, n, e);
    pl.ph[pl.nphase++] = last;
    return pl;
}

// Element offset contributed by register index r in a phase.
constexpr unsigned reg_elem_offset(const PhaseDesc& p, int e, int r) {
    unsigned off = 0;
    for (int q = 0; q < e; ++q)
        if ((r >> q) & 1) off |= 1u << p.rb[q];
    return off;
}

// Every element bit must be butterflied exactly once over the phases.
constexpr bool plan_is_complete(const PlanDesc& pl) {
    unsigned seen = pl.mfma_bits;
    for (int p = 0; p < pl.nphase; ++p) {
        if (seen & pl.ph[p].stages) return false;
        if (pl.ph[p].stages & ~reg_mask(pl.ph[p], pl.e)) return false;
        seen |= pl.ph[p].stages;
    }
    return seen == (1u << pl.n) - 1u;
}

// ---- the matrix-core schedule (bfloat16 I/O, d >= 1024) ---------------------------------------
//
// H_32 applied along five element bits is a 32x32 (+-1) matrix product, which the MFMA unit does
// with exact products and float32 accumulation.  Two such rounds cover bits 0..9:
//   round 1 contracts bits {0,1,2,8,9}: each lane feeds 8 consecutive elements (one 16-byte global
//           vector, bits 0..2), the lane's upper half selects bit 8, the two instructions bit 9;
//           the 32 rows are bits 3..7 (lanes 0..31 read 512 contiguous bytes);
//   round 2 contracts bits {3..7}: the accumulator layout of round 1 has those bits in the register
//           index and the lane's upper half, which is exactly an A-operand layout again.
// After round 2 every lane holds 8 consecutive elements per 16 registers -- the layout it loaded
// in -- so the rounds map the first layout onto itself and leave d/1024 = 2^(t+w) sub-transforms to
// combine: t "tile" bits in registers (2^t MFMA tiles per wave), w bits across the waves of the
// token.  One LDS exchange brings up to 1+t of the wave bits into registers (in place of the first
// layout's upper register bits, whose stages are done); a token of more than 2^(1+t) waves takes a
// second exchange for the rest.
//   first layout : registers (0,1,2, 9, 10..10+t-1), lanes (3..8), waves (10+t..n-1)
//   next layouts : registers (0,1,2, the upper register bits of the previous layout that are not
//                  replaced, the wave bits brought in), lanes (3..8), waves (everything else)
constexpr PlanDesc make_mfma_plan(int n, int t) {
    PlanDesc pl{};
    const int e = 4 + t, v = 3, w = n - 10 - t, c = 1 + t;
    pl.n = n; pl.e = e; pl.v = v; pl.nphase = 0;
    pl.mfma_bits = (1u << 10) - 1u;
    PhaseDesc first{};
    first.rb[0] = 0; first.rb[1] = 1; first.rb[2] = 2; first.rb[3] = 9;
    for (int k = 0; k < t; ++k) first.rb[4 + k] = 10 + k;
    first.stages = 0;
    for (int k = 0; k < t; ++k) first.stages |= 1u << (10 + k);
    fill_thread_bits(first, n, e);
    pl.ph[pl.nphase++] = first;
    PhaseDesc prev = first;
    for (int done = 0; done < w;) {
        const int take = (w - done) < c ? (w - done) : c;
        PhaseDesc next{};
        next.rb[0] = 0; next.rb[1] = 1; next.rb[2] = 2;
        int q = 3;
        for (int k = take; k < c; ++k) next.rb[q++] = prev.rb[3 + k];     // kept upper register bits
        next.stages = 0;
        for (int k = 0; k < take; ++k) {
            const int bit = n - w + done + k;
            next.rb[q++] = bit;
            next.stages |= 1u << bit;
        }
        fill_thread_bits(next, n, e);
        pl.ph[pl.nphase++] = next;
        prev = next;
        done += take;
    }
    return pl;
}

// tiles per wave (log2) used for a given log2 d.  At d = 2^14 the forward pass takes four tiles per
// wave (64 values per thread, one exchange), the backward pass two (32 values per thread, two
// exchanges): its per-thread state (alpha', dalpha, dbeta) does not fit next to 64 values.
constexpr int mfma_log_tiles(int logd, bool backward) {
    return logd <= 10 ? 0 : ((logd >= 14 && !backward) ? 2 : 1);
}

// For a few tokens per launch (one token group per workgroup): as few tiles per wave as the schedule
// allows, i.e. as many waves per token, which shortens each wave's chain of dependent instructions.
constexpr int mfma_log_tiles_few(int logd) { return logd <= 12 ? 0 : 1; }

// ---- rows of 12 * 2^m elements on 2^n = 16 * 2^m slots ----------------------------------------
// Slot index s = (r_hi << 8) | (b << 4) | r_lo  <->  element b * 2^m + (r_hi << 4 | r_lo), m = n - 4:
// the block number b = 0..11 occupies slot bits 4..7, b = 12..15 are padding.  A bit permutation, so
// additive over disjoint bit sets like the LDS maps below.
constexpr unsigned twelve_elem(unsigned s, int n) {
    return (((s >> 4) & 15u) << (n - 4)) | ((s >> 8) << 4) | (s & 15u);
}
constexpr bool twelve_valid(unsigned s) { return ((s >> 6) & 3u) != 3u; }

// P12: symmetric order-12 Hadamard matrix (Paley's second construction over GF(5)), first row and
// column +1.  Bit c of row r's mask is set where P12[r][c] = -1.
// The twelve masks 0x000 0x556 0x3ca 0x96c 0xf22 0x5b8 0xc8e 0x6e4 0x23e 0xb94 0x8f2 0xe58 are packed
// five to a 64-bit word and picked out with shifts: on the GPU a table indexed at run time would be
// a memory load, and the kernels build their matrix operand from this on every launch.
constexpr unsigned paley12_minus_row(unsigned r) {
    const unsigned long long word = r < 5u ? 0x0f2296c3ca556000ull : (r < 10u ? 0x0b9423e6e4c8e5b8ull : 0xe588f2ull);
    const unsigned k = r < 5u ? r : (r < 10u ? r - 5u : r - 10u);
    return (unsigned)(word >> (12u * k)) & 0xfffu;
}
constexpr bool paley12_packing_matches() {
    constexpr unsigned rows[12] = {0x000, 0x556, 0x3ca, 0x96c, 0xf22, 0x5b8,
                                   0xc8e, 0x6e4, 0x23e, 0xb94, 0x8f2, 0xe58};
    for (unsigned r = 0; r < 12u; ++r)
        if (paley12_minus_row(r) != rows[r]) return false;
    return true;
}
static_assert(paley12_packing_matches(), "packed P12 masks");
// Entry of the matrix the second matrix-core round applies along slot bits 3..7 of such a row:
// index m = bit3 + 2 * block;  (-1)^(bit3_in & bit3_out) * P12[block_in][block_out], 0 on padding.
constexpr int twelve_round_entry(unsigned m_in, unsigned m_out) {
    const unsigned bi = m_in >> 1, bo = m_out >> 1;
    if (bi >= 12u || bo >= 12u) return 0;
    const unsigned minus = ((paley12_minus_row(bi) >> bo) ^ (m_in & m_out)) & 1u;
    return minus ? -1 : 1;
}

// ---- LDS address maps -------------------------------------------------------------------------
// Both are linear in the bits of i (phys(a | b) = phys(a) + phys(b) for disjoint a, b) and keep four
// consecutive elements in one aligned 16-byte group.

// Butterfly schedule, padded maps.  The LDS has 32 banks of 4 bytes.
//   8-element vectors (bfloat16 I/O): +4 words every 64 elements keeps the 16-byte-per-lane accesses
//   of the first/last layouts (lane stride 8 words) off each other's banks, +8 words every 256
//   elements does the same for the one-word accesses of the middle layouts (9.4 % of LDS).
//   4-element vectors (fp32 I/O): +4 words every 32 elements and +4 more every 128 elements; the
//   middle layouts' one-word accesses (lanes 2^7 .. 2^10 elements apart) then spread over all banks.
//   Measured at d = 8192: fp32 backward 4 % faster than with the map above; with bfloat16 I/O the
//   bank-conflict cycle counter falls to a third, but the map costs 15.6 % of LDS, which there drops
//   a CU from three resident workgroups to two (forward 12 % slower), so the 8-element case keeps
//   the smaller map.
constexpr unsigned lds_phys_pad(unsigned i, int v) {
    return v == 3 ? i + ((i >> 6) << 2) + ((i >> 8) << 3)
                  : i + ((i >> 5) << 2) + ((i >> 7) << 2);
}
constexpr unsigned lds_words_pad(unsigned d, int v) { return (lds_phys_pad(d - 1, v) + 1 + 3) & ~3u; }

// Matrix-core schedule: both layouts give lane l the 8 elements starting at 8*l (+ multiples of
// 512) as two 16-byte accesses.  Moving element bit 2 above the six lane bits makes each of those
// accesses contiguous across the wave (lane stride 16 bytes): no padding, no bank conflicts.
constexpr unsigned lds_phys_rot(unsigned i) {
    return (i & 3u) | (((i >> 3) & 63u) << 2) | (((i >> 2) & 1u) << 8) | (i & ~511u);
}

}  // namespace wht
