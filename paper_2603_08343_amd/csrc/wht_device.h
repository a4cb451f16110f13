// Device code of the Walsh-Hadamard output layer  y = alpha (.) (H x) + beta  (paper Sec. 4.1,
// Eq. 1) for gfx950: the per-token transform H_raw x (Fig. 2's butterfly stages, scheduled by
// wht_plan.h), the fused affine epilogue, the backward pass with z recomputed, and the fixed-order
// reduction of dalpha / dbeta.  1/sqrt(d) is folded into alpha.  Two schedules share the kernels:
//   - butterfly schedule (float32 I/O, and bfloat16 below d = 1024): every stage is adds/subtracts
//     on register pairs; the token is re-dealt through LDS between groups of stages;
//   - matrix-core schedule (bfloat16 I/O, d >= 1024): ten of the log2(d) stages run as two rounds
//     of 32x32 +-1 products on the MFMA unit (exact products, float32 accumulation), the rest as
//     register butterflies plus one LDS exchange across the waves of a token.
// Widths d = 12 * 2^m (bfloat16, d >= 768; the paper's Table 2 trains d = 768 and 1536 and leaves the
// matrix undefined there) use H_raw = P12 (x) S_{2^m}, P12 a symmetric order-12 Hadamard matrix: the
// matrix-core schedule runs on a row padded to 16 * 2^m slots, with P12 inside the second round's
// +-1 matrix (see MfmaCfg).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "wht_plan.h"

namespace wht {

// ------------------------------------------------------------------------------------------------
// small helpers

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// x, dy are read once and y, dx written once: stream them past the caches (non-temporal).
__device__ __forceinline__ uint4 stream_load16(const void* p) {
    const u32x4 v = __builtin_nontemporal_load(static_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stream_store16(void* p, const uint4& q) {
    const u32x4 v = {q.x, q.y, q.z, q.w};
    __builtin_nontemporal_store(v, static_cast<u32x4*>(p));
}
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// I/O element traits: how one 16-byte global vector maps to float32 registers.
struct IoF32 {
    using elem_t = float;
    static constexpr int kLogVec = 2;   // 4 elements per 16 bytes
    static __device__ __forceinline__ void unpack(const uint4& raw, float* out) {
        out[0] = __uint_as_float(raw.x); out[1] = __uint_as_float(raw.y);
        out[2] = __uint_as_float(raw.z); out[3] = __uint_as_float(raw.w);
    }
    static __device__ __forceinline__ uint4 pack(const float* in) {
        return make_uint4(__float_as_uint(in[0]), __float_as_uint(in[1]),
                          __float_as_uint(in[2]), __float_as_uint(in[3]));
    }
};

struct IoBF16 {
    using elem_t = uint16_t;
    static constexpr int kLogVec = 3;   // 8 elements per 16 bytes
    // bfloat16 is the upper half of binary32: widening is a shift / a mask
    static __device__ __forceinline__ void unpack(const uint4& raw, float* out) {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i]     = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    // round to nearest even (the hardware's packed float32 -> bfloat16 convert)
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
        f32x2 f = {lo, hi};
        bf16x2 b = __builtin_convertvector(f, bf16x2);
        return __builtin_bit_cast(uint32_t, b);
    }
    static __device__ __forceinline__ uint4 pack(const float* in) {
        return make_uint4(pack2(in[0], in[1]), pack2(in[2], in[3]),
                          pack2(in[4], in[5]), pack2(in[6], in[7]));
    }
};

// ------------------------------------------------------------------------------------------------
// per-(d, dtype) configuration

// Butterfly schedule.
template <int LOGD, int LOGE, class Io>
struct Cfg {
    using io = Io;
    static constexpr bool kMfma = false;
    static constexpr int n = LOGD, e = LOGE, v = Io::kLogVec;
    static_assert(v <= e && e <= n && e <= kMaxRegBits, "bad tile");
    static constexpr PlanDesc plan = make_plan(n, e, v);
    static_assert(plan_is_complete(plan), "every butterfly stage must run exactly once");
    static constexpr int P = plan.nphase;
    static constexpr int D = 1 << n;
    static constexpr int E = 1 << e;            // values per thread
    static constexpr int V = 1 << v;            // elements per 16-byte vector
    static constexpr int NV = E / V;            // 16-byte vectors per thread
    static constexpr int TPT = 1 << (n - e);    // threads per token
    static constexpr int BT = TPT > 256 ? TPT : 256;   // threads per workgroup
    static constexpr int G = BT / TPT;          // tokens per workgroup pass
    static constexpr bool kTwelve = false;
    // persistent-grid size in workgroups per CU (measured optima, N = 16384..32768 tokens)
    static constexpr int kFwdGroupsPerCU = v == 2 ? (n >= 13 ? 8 : 4) : (n <= 9 ? 2 : 8);
    static constexpr int kBwdGroupsPerCU = v == 2 ? 1 : 2;
    static constexpr int kFwdCluster = 0, kFwdClusterResid = 0;     // see MfmaCfg
    static constexpr bool kBwdTeams = false;    // see MfmaCfg
    static constexpr int kRow = D;              // elements per row in memory
    static constexpr unsigned real(unsigned i) { return i; }
    static constexpr bool valid(unsigned) { return true; }
    static constexpr unsigned phys(unsigned i) { return lds_phys_pad(i, v); }
    static constexpr unsigned kTokenWords = lds_words_pad(D, v);
    static constexpr unsigned kExchangeBytes = (P > 1 || G > 1) ? G * kTokenWords * 4u : 16u;
    static constexpr unsigned kStageBytes = BT * NV * 16u;          // one tensor's token group, as stored
    static constexpr unsigned kLdsBytes = kExchangeBytes + kStageBytes;              // forward
    static constexpr unsigned kLdsBytesBackward = kExchangeBytes + 2u * kStageBytes; // x and dy
    static_assert(kLdsBytesBackward <= 160u * 1024u, "token group does not fit LDS");
};

// Matrix-core schedule (bfloat16 I/O, d >= 1024): 2^LOGT MFMA tiles of 1024 elements per wave.
//
// TWELVE: the row in memory has 12 * 2^m elements (m = LOGD - 4) and the schedule runs on 2^LOGD
// "slots".  Slot index s = (r_hi << 8) | (b << 4) | r_lo  <->  element b * 2^m + (r_hi << 4 | r_lo):
// the block number b = 0..11 sits in slot bits 4..7 (b = 12..15 are empty slots, held as zeros and
// never loaded or stored), so that the second round, which contracts slot bits 3..7, sees the pair
// (element bit 3, block) and applies  P12 (x) H_2  there; every other slot bit is an ordinary
// Sylvester bit.  Bits 6 and 7 are lane bits in both memory layouts, so a slot's validity is a
// property of the lane: lanes 24..31 and 56..63 of every wave sit out the loads and stores, and
// per instruction the others touch 64 contiguous bytes of every block, as two 32-byte lane pairs
// (l, l+1) and (l+32, l+33).
template <int LOGD, int LOGT, bool TWELVE = false>
struct MfmaCfg {
    using io = IoBF16;
    static constexpr bool kMfma = true;
    static constexpr bool kTwelve = TWELVE;
    static constexpr int n = LOGD, t = LOGT, e = 4 + LOGT, v = 3;
    static constexpr int w = n - 10 - t;        // log2(waves per token)
    static_assert(n >= 10 && w >= 0 && w <= 2 * (1 + t) && e <= kMaxRegBits, "bad tile");
    static constexpr PlanDesc plan = make_mfma_plan(n, t);
    static_assert(plan_is_complete(plan), "every stage must run exactly once");
    static constexpr int P = plan.nphase;
    static constexpr int D = 1 << n;
    static constexpr int E = 1 << e;
    static constexpr int V = 8;
    static constexpr int NV = E / V;
    static constexpr int T = 1 << t;            // MFMA tiles per wave
    static constexpr int TPT = 1 << (n - e);
    static_assert(TPT >= 64, "a token occupies whole waves");
    static constexpr int BT = TPT > 256 ? TPT : 256;
    static constexpr int G = BT / TPT;
    // persistent-grid size in workgroups per CU (measured optima at N = 32768 tokens: more
    // workgroups than this only add concurrent streams to the memory system)
    static constexpr int kFwdGroupsPerCU = 2;
    // the full backward of a schedule with one LDS exchange runs on three teams of waves
    // (backward_teams_kernel), one workgroup per CU
    static constexpr bool kBwdTeams = plan.nphase == 2 && 3 * BT <= 1024;
    static constexpr int kBwdGroupsPerCU = kBwdTeams ? 1 : (TWELVE ? (n == 11 ? 1 : 2) : ((n == 11 || n >= 13) ? 1 : 2));
    // Forward: workgroups per cluster (0 = one interleave over the whole grid).  With every
    // workgroup in one moving window of rows, the read stream and the write stream keep a fixed
    // address distance, and for about 40 % of the distances y - x (period 128 MiB, and again 512 KiB)
    // the kernel runs 8..29 % slower at d >= 4096 -- DRAM bank conflicts between the two streams.
    // Four windows spread over the tensor take the worst case from +29 % to +11 % and improve the
    // mean over all distances, for +1.5 % in the best case.  Rows of 4 KiB and less show no such
    // dependence and keep the plain interleave.
    static constexpr int kFwdCluster = n >= 12 ? 128 : 0;
    // with the residual as a third stream two windows measured best (mean 263 us against 274 us
    // with four and 268 us with one, d = 8192)
    static constexpr int kFwdClusterResid = n >= 12 ? 256 : 0;
    static constexpr int kRow = TWELVE ? 3 * (D / 4) : D;       // elements per row in memory
    static constexpr unsigned real(unsigned s) {                // slot index -> element index
        return TWELVE ? twelve_elem(s, n) : s;
    }
    static constexpr bool valid(unsigned s) { return !TWELVE || twelve_valid(s); }
    static_assert(!TWELVE || ((reg_mask(plan.ph[0], e) | reg_mask(plan.ph[P - 1], e)) & 0xC0u) == 0,
                  "block bits 6 and 7 must be lane bits in the memory layouts");
    static constexpr unsigned phys(unsigned i) { return lds_phys_rot(i); }
    static constexpr unsigned kTokenWords = D;
    static constexpr unsigned kExchangeBytes = (P > 1 || G > 1) ? G * kTokenWords * 4u : 16u;
    static constexpr unsigned kStageBytes = BT * NV * 16u;          // one tensor's token group, as stored
    static constexpr unsigned kLdsBytes = kExchangeBytes + kStageBytes;              // forward
    static constexpr unsigned kLdsBytesBackward = kExchangeBytes + 2u * kStageBytes; // x and dy
    static_assert(kLdsBytesBackward <= 160u * 1024u, "token group does not fit LDS");
};

// Element offset of thread t (within its token) in phase PH.
template <class C, int PH>
__device__ __forceinline__ unsigned thread_elem_offset(unsigned t) {
    unsigned off = 0;
    static_for<0, C::n - C::e>([&](auto k) {
        constexpr int K = decltype(k)::value;
        off |= ((t >> K) & 1u) << C::plan.ph[PH].tb[K];
    });
    return off;
}

// Butterfly stages of phase PH, all in registers: (a, b) -> (a + b, a - b) on register pairs.
template <class C, int PH>
__device__ __forceinline__ void run_stages(float (&r)[C::E]) {
    static_for<0, C::e>([&](auto q) {
        constexpr int Q = decltype(q)::value;
        constexpr int bit = C::plan.ph[PH].rb[Q];
        if constexpr ((C::plan.ph[PH].stages >> bit) & 1u) {
            static_for<0, C::E>([&](auto i) {
                constexpr int I = decltype(i)::value;
                if constexpr (!((I >> Q) & 1)) {
                    const float a = r[I], b = r[I | (1 << Q)];
                    r[I] = a + b;
                    r[I | (1 << Q)] = a - b;
                }
            });
        }
    });
}

// Debug build (WHT_POISON_LDS, used by csrc/poison_check.hip only): a thread that has read its
// values from an exchange region or from its own stage slot overwrites them with NaN.  A read that
// comes too early -- before the data it is meant to see has been written or has landed, i.e. a
// missing barrier or a missing wait -- then returns NaN instead of last iteration's plausible
// values, and the comparison against the oracle fails loudly.
#ifdef WHT_POISON_LDS
constexpr bool kPoisonLds = true;
#else
constexpr bool kPoisonLds = false;
#endif

template <class C, int PH>
constexpr bool phase_is_vec4() { return C::plan.ph[PH].rb[0] == 0 && C::plan.ph[PH].rb[1] == 1; }

// Registers <-> LDS in the layout of phase PH.  `tok` points at this token's LDS region plus the
// thread's own (runtime) offset; register offsets are compile-time immediates.
template <class C, int PH>
__device__ __forceinline__ void lds_put(const float (&r)[C::E], float* tok) {
    if constexpr (phase_is_vec4<C, PH>()) {
        static_for<0, C::E / 4>([&](auto i) {
            constexpr int I = decltype(i)::value * 4;
            constexpr unsigned off = C::phys(reg_elem_offset(C::plan.ph[PH], C::e, I));
            *reinterpret_cast<float4*>(tok + off) = make_float4(r[I], r[I + 1], r[I + 2], r[I + 3]);
        });
    } else {
        static_for<0, C::E>([&](auto i) {
            constexpr int I = decltype(i)::value;
            constexpr unsigned off = C::phys(reg_elem_offset(C::plan.ph[PH], C::e, I));
            tok[off] = r[I];
        });
    }
}

template <class C, int PH>
__device__ __forceinline__ void lds_get(float (&r)[C::E], const float* tok) {
    if constexpr (phase_is_vec4<C, PH>()) {
        static_for<0, C::E / 4>([&](auto i) {
            constexpr int I = decltype(i)::value * 4;
            constexpr unsigned off = C::phys(reg_elem_offset(C::plan.ph[PH], C::e, I));
            const float4 q = *reinterpret_cast<const float4*>(tok + off);
            r[I] = q.x; r[I + 1] = q.y; r[I + 2] = q.z; r[I + 3] = q.w;
        });
    } else {
        static_for<0, C::E>([&](auto i) {
            constexpr int I = decltype(i)::value;
            constexpr unsigned off = C::phys(reg_elem_offset(C::plan.ph[PH], C::e, I));
            r[I] = tok[off];
        });
    }
    if constexpr (kPoisonLds) {
        const float nan = __uint_as_float(0x7fc00000u);
        static_for<0, C::E>([&](auto i) {
            constexpr int I = decltype(i)::value;
            constexpr unsigned off = C::phys(reg_elem_offset(C::plan.ph[PH], C::e, I));
            const_cast<float*>(tok)[off] = nan;
        });
    }
}

// Per-thread constants: LDS word offset of the thread in every phase, element offset in the first
// and last phase (the global-memory layouts).
template <class C>
struct ThreadMap {
    unsigned lds_off[kMaxPhases];
    unsigned first_elem, last_elem;     // offset within the row in memory
    bool first_ok, last_ok;             // false for a thread whose slots are padding (12 * 2^m rows)
    __device__ __forceinline__ void init(unsigned t, unsigned slot) {
        static_for<0, C::P>([&](auto p) {
            constexpr int PH = decltype(p)::value;
            lds_off[PH] = slot * C::kTokenWords + C::phys(thread_elem_offset<C, PH>(t));
        });
        const unsigned f = thread_elem_offset<C, 0>(t), l = thread_elem_offset<C, C::P - 1>(t);
        first_elem = C::real(f);
        last_elem = C::real(l);
        first_ok = C::valid(f);
        last_ok = C::valid(l);
    }
};

// H_raw applied to the 2^n values spread over the token's threads.
//   FORWARD_ORDER: registers enter in the first phase's layout and leave in the last phase's;
//   otherwise the phases run in reverse (enter in the last layout, leave in the first) -- the
//   backward pass uses this so that dy can be consumed in the layout z was produced in.
// Ends with a workgroup barrier when LDS was used, so the caller may reuse LDS at once.
// Workgroup barrier for the LDS exchange.  __syncthreads() carries a release/acquire fence that
// makes the wave wait for *all* its outstanding memory operations -- including the prefetches in
// flight and the stores of the previous token, which have nothing to do with the exchange.  The
// exchange only needs this wave's LDS writes to have completed (lgkmcnt) before the barrier.
__device__ __forceinline__ void exchange_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <class C, bool FORWARD_ORDER, bool TRAILING_BARRIER>
__device__ __forceinline__ void transform(float (&r)[C::E], float* lds, const ThreadMap<C>& tm) {
    static_for<0, C::P>([&](auto s) {
        constexpr int S = decltype(s)::value;
        constexpr int PH = FORWARD_ORDER ? S : C::P - 1 - S;
        if constexpr (S > 0) lds_get<C, PH>(r, lds + tm.lds_off[PH]);
        run_stages<C, PH>(r);
        if constexpr (S + 1 < C::P) {
            // a middle phase rewrites exactly the words it read, so only the hand-over to the
            // next layout needs the barrier
            lds_put<C, PH>(r, lds + tm.lds_off[PH]);
            exchange_barrier();
        }
    });
    // The next write into the exchange region must not overtake other waves' reads of this one.
    // When the next transform runs in the opposite order (the backward kernel alternates), its
    // first write goes, thread by thread, to exactly the words this thread has just read, and no
    // barrier is needed; a kernel that only runs forward-order transforms needs it.
    if constexpr (C::P > 1 && TRAILING_BARRIER) exchange_barrier();
}

// Global -> LDS staging -> registers.  x and dy are fetched with LDS-direct loads (the data goes
// from memory into LDS without passing through registers), a whole iteration before they are used,
// so that tens of KiB per workgroup are in flight at all times at no register cost.  An LDS-direct
// load of 16 bytes writes lane l's vector to (wave-uniform base) + 16*l: every wave owns a private
// 1 KiB slot per vector, reads back exactly what it fetched, and needs no workgroup barrier --
// only its own vmcnt (loads return in issue order) and lgkmcnt waits, which are written out here
// because the compiler does not track the dependence between an LDS-direct load and a later LDS read.
constexpr int kStreamPolicy = 2;   // cache-policy operand of the load: "nt" (read once, do not retain)
typedef const __attribute__((address_space(1))) void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_ptr;

template <class C, int PH>
__device__ __forceinline__ void stage_issue(unsigned char* wave_slot, const typename C::io::elem_t* row,
                                            unsigned thread_elem, bool ok) {
    static_for<0, C::NV>([&](auto c) {
        constexpr int Cc = decltype(c)::value;
        constexpr unsigned off = C::real(reg_elem_offset(C::plan.ph[PH], C::e, Cc * C::V));
        if constexpr (C::kTwelve) {
            // padding lanes fetch nothing (their stage slots are never used); the others fetch
            // 32-byte pieces, two instructions per 128-byte line: cached, so the line is read once
            if (ok)
                __builtin_amdgcn_global_load_lds((global_cptr)(row + thread_elem + off),
                                                 (lds_ptr)(wave_slot + Cc * 1024), 16, 0, 0);
        } else {
            __builtin_amdgcn_global_load_lds((global_cptr)(row + thread_elem + off),
                                             (lds_ptr)(wave_slot + Cc * 1024), 16, 0, kStreamPolicy);
        }
    });
}

// Read the staged vectors back.  Written as inline assembly on purpose: for a compiler-visible
// LDS load the waitcnt insertion would wait for *every* LDS-direct load in flight (vmcnt(0)),
// including the next group's prefetch issued moments ago.  Which loads must have landed is known
// here (wait_vmem below, issued by the caller first); the reads' own completion is awaited inside
// this function, with the values tied to the wait so that no use can be scheduled before it.
__device__ __forceinline__ unsigned lds_byte_address(const void* p) {
    return (unsigned)(size_t)(const __attribute__((address_space(3))) unsigned char*)p;
}

//   OWN: the slot was filled by this wave's own loads and nobody else reads it (poisoned after the
//   read in the debug build); false for a slot that another wave fetched or also reads.
template <class C, bool OWN = true>
__device__ __forceinline__ void stage_read(uint4 (&raw)[C::NV], const unsigned char* wave_slot) {
    static_assert(C::NV == 1 || C::NV == 2 || C::NV == 4 || C::NV == 8, "unexpected vector count");
    const unsigned addr = lds_byte_address(wave_slot) + (threadIdx.x & 63u) * 16u;
    u32x4 v[C::NV];
#pragma unroll
    for (int c = 0; c < C::NV; ++c) {
        const unsigned a = addr + c * 1024;
        asm volatile("ds_read_b128 %0, %1" : "=&v"(v[c]) : "v"(a) : "memory");
    }
    if constexpr (C::NV == 1)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v[0]) : : "memory");
    else if constexpr (C::NV == 2)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v[0]), "+v"(v[1]) : : "memory");
    else if constexpr (C::NV == 4)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]) : : "memory");
    else
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7])
                     : : "memory");
#pragma unroll
    for (int c = 0; c < C::NV; ++c) raw[c] = make_uint4(v[c].x, v[c].y, v[c].z, v[c].w);
    if constexpr (kPoisonLds && OWN) {
        const u32x4 nan = {0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u};   // NaN as bf16 pairs and as f32
#pragma unroll
        for (int c = 0; c < C::NV; ++c) {
            const unsigned a = addr + c * 1024;
            asm volatile("ds_write_b128 %0, %1" : : "v"(a), "v"(nan) : "memory");
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
}

// Padding lanes of a 12 * 2^m row read stale LDS: replace it by zeros (the padding's value).
template <class C>
__device__ __forceinline__ void zero_padding(uint4 (&raw)[C::NV], bool ok) {
    if constexpr (C::kTwelve) {
#pragma unroll
        for (int c = 0; c < C::NV; ++c)
            if (!ok) raw[c] = make_uint4(0u, 0u, 0u, 0u);
    }
}

// Wait until at most PENDING of this wave's vector-memory operations are outstanding.
template <int PENDING>
__device__ __forceinline__ void wait_vmem() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PENDING) : "memory");
}
template <class C>
__device__ __forceinline__ void unpack_all(float (&r)[C::E], const uint4 (&raw)[C::NV]) {
    static_for<0, C::NV>([&](auto c) {
        constexpr int Cc = decltype(c)::value;
        C::io::unpack(raw[Cc], &r[Cc * C::V]);
    });
}

// STREAM: non-temporal stores.  Rows of 12 * 2^m elements are written in 32-byte pieces: there
// plain stores, which L2 merges into whole lines, are used instead (17 % faster in the forward
// kernel at d = 6144, 6 % in the backward kernel, and no partial-line write traffic).
template <class C, int PH, bool STREAM = true>
__device__ __forceinline__ void global_put(const float (&r)[C::E], typename C::io::elem_t* row,
                                           unsigned thread_elem, bool active) {
    static_for<0, C::NV>([&](auto c) {
        constexpr int Cc = decltype(c)::value;
        constexpr unsigned off = C::real(reg_elem_offset(C::plan.ph[PH], C::e, Cc * C::V));
        if (active) {
            if constexpr (STREAM) stream_store16(row + thread_elem + off, C::io::pack(&r[Cc * C::V]));
            else *reinterpret_cast<uint4*>(row + thread_elem + off) = C::io::pack(&r[Cc * C::V]);
        }
    });
}

// float32 parameter vector -> registers in the layout of phase PH, times `scale`.
template <class C, int PH>
__device__ __forceinline__ void param_get(float (&r)[C::E], const float* p, unsigned thread_elem,
                                          bool ok, float scale) {
    // Padding lanes of a 12 * 2^m row read block 0 instead (in bounds) and scale it to zero: a load
    // under a per-lane condition costs the compiler a second copy of every parameter register.
    const unsigned base = (!C::kTwelve || ok) ? thread_elem : 0u;
    const float sc = (!C::kTwelve || ok) ? scale : 0.0f;
    static_for<0, C::E / 4>([&](auto i) {
        constexpr int I = decltype(i)::value * 4;
        constexpr unsigned off = C::real(reg_elem_offset(C::plan.ph[PH], C::e, I));
        const float4 q = *reinterpret_cast<const float4*>(p + base + off);
        r[I] = q.x * sc; r[I + 1] = q.y * sc; r[I + 2] = q.z * sc; r[I + 3] = q.w * sc;
    });
}

// ------------------------------------------------------------------------------------------------
// matrix-core rounds: H_32 along five element bits as a 32x32x32 product with a +-1 matrix
//
// v_mfma_f32_32x32x16_bf16 operand layout (two instructions cover K = 32):
//   A[i][k]: lane = i + 32*(k/8 % 2), element k%8 of the lane's 8 bf16, instruction k/16
//   B[k][j]: lane = j + 32*(k/8 % 2), element k%8, instruction k/16
//   D[i][j]: lane = j + 32*(i/4 % 2), register 4*(i/8) + i%4
// With B[k][j] = (-1)^popcount(k & swap23(j)) (bits 2 and 3 of j exchanged) the accumulator of a
// round is again an A operand for the next one -- rows <-> the previous round's outputs, K <-> the
// previous round's rows -- and after two rounds each lane holds, in register order, the 8 + 8
// consecutive elements it loaded.

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct HadamardB {
    bf16x8 k_lo, k_hi;      // B operand of the first / second K-half
};

__device__ __forceinline__ HadamardB make_hadamard_b() {
    const unsigned lane = threadIdx.x & 63u;
    const unsigned j = lane & 31u, kg = lane >> 5;
    const unsigned js = (j & 0x13u) | ((j & 4u) << 1) | ((j & 8u) >> 1);
    uint32_t w[2][4];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const unsigned k0 = (2u * p) | (kg << 3) | ((unsigned)half << 4), k1 = k0 | 1u;
            const uint32_t lo = (__popc(k0 & js) & 1) ? 0xBF80u : 0x3F80u;     // bf16 -1 : +1
            const uint32_t hi = (__popc(k1 & js) & 1) ? 0xBF80u : 0x3F80u;
            w[half][p] = lo | (hi << 16);
        }
    HadamardB b;
    b.k_lo = __builtin_bit_cast(bf16x8, make_uint4(w[0][0], w[0][1], w[0][2], w[0][3]));
    b.k_hi = __builtin_bit_cast(bf16x8, make_uint4(w[1][0], w[1][1], w[1][2], w[1][3]));
    return b;
}

// Second-round matrix for rows of 12 * 2^m elements.  The round contracts slot bits 3..7: bit 3 is
// an ordinary Sylvester bit, bits 4..7 are the block number, so with m = bit3 + 2 * block the
// matrix is  M[m_in][m_out] = (-1)^(bit3_in & bit3_out) * P12[block_in][block_out], and zero when
// either block is one of the four empty ones.  In the operand layout above the second round's K
// index arrives with bits 2 and 3 exchanged and its column index in natural order, hence
// B[k][j] = M[swap23(k)][j], M = twelve_round_entry (wht_plan.h).
__device__ __forceinline__ HadamardB make_paley_b(const HadamardB& sylvester) {
    const unsigned lane = threadIdx.x & 63u;
    const unsigned j = lane & 31u, kg = lane >> 5;
    uint32_t w[2][4];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            uint32_t pair = 0;
#pragma unroll
            for (int odd = 0; odd < 2; ++odd) {
                const unsigned k = (2u * p) | (unsigned)odd | (kg << 3) | ((unsigned)half << 4);
                const unsigned m_in = (k & 0x13u) | ((k & 4u) << 1) | ((k & 8u) >> 1);
                const int sign = twelve_round_entry(m_in, j);
                const uint32_t entry = sign == 0 ? 0u : (sign < 0 ? 0xBF80u : 0x3F80u);   // bf16 0, -1, +1
                pair |= entry << (16 * odd);
            }
            w[half][p] = pair;
        }
    HadamardB b = sylvester;
    b.k_lo = __builtin_bit_cast(bf16x8, make_uint4(w[0][0], w[0][1], w[0][2], w[0][3]));
    b.k_hi = __builtin_bit_cast(bf16x8, make_uint4(w[1][0], w[1][1], w[1][2], w[1][3]));
    return b;
}

// One round on bfloat16 data straight from memory: products and sums are exact up to the
// accumulator's float32 rounding.
__device__ __forceinline__ f32x16 hadamard_round_bf16(const uint4& a_lo, const uint4& a_hi,
                                                      const HadamardB& b) {
    f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_lo), b.k_lo, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_hi), b.k_hi, acc, 0, 0, 0);
    return acc;
}

// One round on float32 data: each value is split into bf16 hi + bf16 lo (hi = RNE(v), lo =
// RNE(v - hi); v - hi is exact, so |v - hi - lo| <= 2^-17 |v|) and both parts go through the same
// +-1 product, accumulated in float32.  v - hi is formed with plain vector instructions (widen hi by
// a shift / a mask, subtract): the bf16 dot-product instruction would do it in one, but it executes
// on the matrix pipeline and stalls behind the rounds' own MFMAs (measured: 20 cycles per dot
// instruction next to back-to-back MFMAs, against 4.4 alone).
__device__ __forceinline__ f32x16 hadamard_round_f32(const float* v, const HadamardB& b) {
    uint32_t hi[8], lo[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const uint32_t h = IoBF16::pack2(v[2 * p], v[2 * p + 1]);
        const float l0 = v[2 * p] - __uint_as_float(h << 16);
        const float l1 = v[2 * p + 1] - __uint_as_float(h & 0xffff0000u);
        hi[p] = h;
        lo[p] = IoBF16::pack2(l0, l1);
    }
    f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const bf16x8 lo0 = __builtin_bit_cast(bf16x8, make_uint4(lo[0], lo[1], lo[2], lo[3]));
    const bf16x8 lo1 = __builtin_bit_cast(bf16x8, make_uint4(lo[4], lo[5], lo[6], lo[7]));
    const bf16x8 hi0 = __builtin_bit_cast(bf16x8, make_uint4(hi[0], hi[1], hi[2], hi[3]));
    const bf16x8 hi1 = __builtin_bit_cast(bf16x8, make_uint4(hi[4], hi[5], hi[6], hi[7]));
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo0, b.k_lo, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo1, b.k_hi, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi0, b.k_lo, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi1, b.k_hi, acc, 0, 0, 0);
    return acc;
}

// Both rounds on every tile of the thread: bits 0..9 of the element index.  b is the Sylvester
// matrix; b2, the second round's matrix, is the same except for rows of 12 * 2^m elements.  Round 1 of every tile
// is issued before any round 2, so that one tile's split has the other tile's matrix instructions
// to overlap with.  (Explicit MFMA/VALU interleave hints on top of this measured no gain.)
//   from raw bfloat16 (the forward input x): round 1 needs no split
template <class C>
__device__ __forceinline__ void mfma_rounds_from_bf16(float (&r)[C::E], const uint4 (&raw)[C::NV],
                                                      const HadamardB& b, const HadamardB& b2) {
    f32x16 d1[C::T];
    static_for<0, C::T>([&](auto tile) {
        constexpr int Tl = decltype(tile)::value;
        d1[Tl] = hadamard_round_bf16(raw[2 * Tl], raw[2 * Tl + 1], b);
    });
    static_for<0, C::T>([&](auto tile) {
        constexpr int Tl = decltype(tile)::value;
        float v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = d1[Tl][i];
        const f32x16 d2 = hadamard_round_f32(v, b2);
#pragma unroll
        for (int i = 0; i < 16; ++i) r[16 * Tl + i] = d2[i];
    });
}
//   from float32 registers in the first layout (the backward pass's alpha' (.) dy)
template <class C>
__device__ __forceinline__ void mfma_rounds_from_f32(float (&r)[C::E], const HadamardB& b,
                                                     const HadamardB& b2) {
    f32x16 d1[C::T];
    static_for<0, C::T>([&](auto tile) {
        constexpr int Tl = decltype(tile)::value;
        d1[Tl] = hadamard_round_f32(&r[16 * Tl], b);
    });
    static_for<0, C::T>([&](auto tile) {
        constexpr int Tl = decltype(tile)::value;
        float v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = d1[Tl][i];
        const f32x16 d2 = hadamard_round_f32(v, b2);
#pragma unroll
        for (int i = 0; i < 16; ++i) r[16 * Tl + i] = d2[i];
    });
}

// raw x[tok] (first layout) -> H_raw x in the last layout, whichever schedule C is.
template <class C, bool TRAILING_BARRIER>
__device__ __forceinline__ void transform_from_raw(float (&r)[C::E], const uint4 (&raw)[C::NV],
                                                   float* lds, const ThreadMap<C>& tm,
                                                   const HadamardB& b, const HadamardB& b2) {
    if constexpr (C::kMfma) mfma_rounds_from_bf16<C>(r, raw, b, b2);
    else                    unpack_all<C>(r, raw);
    transform<C, true, TRAILING_BARRIER>(r, lds, tm);
}

// registers in the last layout -> H_raw (.) in the first layout.
template <class C, bool TRAILING_BARRIER = false>
__device__ __forceinline__ void transform_back(float (&r)[C::E], float* lds, const ThreadMap<C>& tm,
                                               const HadamardB& b, const HadamardB& b2) {
    transform<C, false, TRAILING_BARRIER>(r, lds, tm);
    if constexpr (C::kMfma) mfma_rounds_from_f32<C>(r, b, b2);
}

template <class C>
__device__ __forceinline__ float inv_sqrt_d() {
    if constexpr (C::kTwelve) {
        // d = 3 * 2^(n-2): 1/sqrt(3) or 1/sqrt(6), rounded once, times a power of two
        return ((C::n - 2) % 2 == 0) ? 0.57735026918962576451f / float(1 << ((C::n - 2) / 2))
                                     : 0.40824829046386301637f / float(1 << ((C::n - 2) / 2));
    }
    // exact power of two for even log2 d; one rounding of 1/sqrt(2) * 2^-k otherwise
    return (C::n % 2 == 0) ? 1.0f / float(1 << (C::n / 2))
                           : 0.70710678118654752440f / float(1 << (C::n / 2));
}

// ------------------------------------------------------------------------------------------------
// Kernels.  A workgroup holds G token slots of TPT threads each and strides over token groups
// (persistent grid).  Inputs of group k+1 are in flight (LDS-direct loads) while group k is
// computed.  A ragged last group re-reads the last token (clamped row) and masks its stores.

template <class C>
struct Walker {
    int64_t N, groups;
    unsigned slot;
    __device__ __forceinline__ int64_t token(int64_t grp) const { return grp * C::G + slot; }
    __device__ __forceinline__ int64_t row(int64_t grp) const {       // clamped: always a valid row
        const int64_t tok = token(grp);
        return tok < N ? tok : N - 1;
    }
};

// sumsq[tok] = sum of the token's r[i]^2 (the values as they stand, before rounding for the store):
// each thread squares its values, the lanes of a token add up by butterfly shuffles, and a token that
// spans several waves adds the wave sums through `wave_sums` (one float per wave of the workgroup)
// in a fixed order, behind one workgroup barrier that every wave passes.
template <class C>
__device__ __forceinline__ void token_sumsq(const float (&r)[C::E], float* wave_sums, float* __restrict__ sumsq,
                                            int64_t tok, int64_t N, unsigned t, unsigned slot, bool lane_ok) {
    float sq = 0.0f;
#pragma unroll
    for (int i = 0; i < C::E; ++i) sq = fmaf(r[i], r[i], sq);
    if (C::kTwelve && !lane_ok) sq = 0.0f;                  // padding lanes hold no elements
    constexpr int kLanes = C::TPT < 64 ? C::TPT : 64;       // lanes of one wave that share a token
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) sq += __shfl_xor(sq, off);
    if constexpr (C::TPT <= 64) {
        if (t == 0 && tok < N) sumsq[tok] = sq;
    } else {
        constexpr int kWaves = C::TPT / 64;                 // waves per token
        if ((threadIdx.x & 63u) == 0) wave_sums[threadIdx.x >> 6] = sq;
        exchange_barrier();
        if (t == 0 && tok < N) {
            float total = 0.0f;
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) total += wave_sums[slot * kWaves + wv];
            sumsq[tok] = total;
        }
    }
}

// forward:  y = (alpha / sqrt d) (.) (H_raw x) + beta      [+ resid when RESID]
//
// Per iteration k (x(k) [and resid(k)] have landed in their stages):
//   raw <- stage;  issue x(k+1) -> stage;  transform raw;  affine;  wait for everything pending;
//   store y(k).
// The one wait sits just before the stores of y(k): all it can be waiting for is x(k+1), issued a
// whole transform earlier, and the stores of y(k-1), a whole iteration old.  (Loads and stores may
// complete out of order with respect to each other, so a counted wait is only safe when nothing
// but older loads is pending; waiting here, before the new stores, keeps it that way.)
// RESID fuses the attention block's residual add into the epilogue: resid is one more staged
// stream, fetched in the layout y is stored in.
// STATS (with RESID) also writes sumsq[token] = sum_j y[token][j]^2, taken from the float32 values
// before they are rounded for the store: the statistic of an RMS normalisation that follows the
// residual stream.  Each thread squares its values, the lanes of a token add up by butterfly
// shuffles, and a token that spans several waves adds the wave sums through LDS in a fixed order
// (one more workgroup barrier per token; the next write to that LDS array is behind the next
// token's exchange barriers, so nothing else is needed).
template <class C, bool RESID, bool STATS = false>
__global__ __launch_bounds__(C::BT) void forward_kernel(const typename C::io::elem_t* x,
                                                        const float* __restrict__ alpha,
                                                        const float* __restrict__ beta,
                                                        const typename C::io::elem_t* resid,
                                                        typename C::io::elem_t* y,
                                                        float* __restrict__ sumsq,
                                                        int64_t N, int cluster) {
    static_assert(!STATS || RESID, "the statistic belongs to the residual-stream output");
    static_assert(!STATS || C::TPT <= 64 || C::P > 1, "a token of several waves has an exchange");
    __shared__ float wave_sums[STATS ? C::BT / 64 : 1];
    // separate LDS objects: the compiler can then tell that the exchange region's accesses never
    // alias an LDS-direct load in flight, and does not wait for the prefetch before them
    __shared__ __align__(16) float lds[C::kExchangeBytes / 4];
    __shared__ __align__(16) unsigned char stage_buf[C::kStageBytes];
    __shared__ __align__(16) unsigned char stage_r_buf[RESID ? C::kStageBytes : 16];
    constexpr int LAST = C::P - 1;
    const unsigned t = threadIdx.x % C::TPT;
    Walker<C> wk{N, (N + C::G - 1) / C::G, threadIdx.x / C::TPT};
    ThreadMap<C> tm;
    tm.init(t, wk.slot);
    HadamardB hb{}, hbp{};
    if constexpr (C::kMfma) hb = make_hadamard_b();
    if constexpr (C::kTwelve) hbp = make_paley_b(hb);
    const HadamardB& hb2 = C::kTwelve ? hbp : hb;
    unsigned char* stage = stage_buf + (threadIdx.x >> 6) * (C::NV * 1024);
    unsigned char* stage_r = stage_r_buf + (RESID ? (threadIdx.x >> 6) * (C::NV * 1024) : 0);

    // Token groups are dealt to clusters of `cluster` consecutive workgroups: the token groups are
    // cut into gridDim.x / cluster contiguous regions, and a cluster walks its region interleaved
    // (workgroup j of the cluster takes groups j, j + cluster, ...).  cluster = gridDim.x is the
    // plain interleave over the whole grid.
    const int64_t step = cluster;
    const int64_t nclus = gridDim.x / cluster, clus = blockIdx.x / cluster;
    const int64_t per = (wk.groups + nclus - 1) / nclus;
    int64_t grp = clus * per + blockIdx.x % cluster;
    const int64_t grp_end = (clus + 1) * per < wk.groups ? (clus + 1) * per : wk.groups;
    // first token's fetch goes out before anything else; the parameters load in its shadow
    if (grp < grp_end) {
        stage_issue<C, 0>(stage, x + wk.row(grp) * C::kRow, tm.first_elem, tm.first_ok);
        if constexpr (RESID)
            stage_issue<C, LAST>(stage_r, resid + wk.row(grp) * C::kRow, tm.last_elem, tm.last_ok);
    }

    float a[C::E], b[C::E];
    param_get<C, LAST>(a, alpha, tm.last_elem, tm.last_ok, inv_sqrt_d<C>());
    param_get<C, LAST>(b, beta, tm.last_elem, tm.last_ok, 1.0f);
    wait_vmem<0>();
    for (; grp < grp_end; grp += step) {
        const bool more = grp + step < grp_end;
        uint4 raw[C::NV], rraw[RESID ? C::NV : 1];
        stage_read<C>(raw, stage);
        zero_padding<C>(raw, tm.first_ok);
        if constexpr (RESID) stage_read<C>(rraw, stage_r);
        if (more) {
            stage_issue<C, 0>(stage, x + wk.row(grp + step) * C::kRow, tm.first_elem, tm.first_ok);
            if constexpr (RESID)
                stage_issue<C, LAST>(stage_r, resid + wk.row(grp + step) * C::kRow, tm.last_elem, tm.last_ok);
        }
        float r[C::E];
        transform_from_raw<C, true>(r, raw, lds, tm, hb, hb2);
        if constexpr (RESID) {
            float res[C::E];
            unpack_all<C>(res, rraw);
#pragma unroll
            for (int i = 0; i < C::E; ++i) r[i] = res[i] + fmaf(r[i], a[i], b[i]);
        } else {
#pragma unroll
            for (int i = 0; i < C::E; ++i) r[i] = fmaf(r[i], a[i], b[i]);
        }
        const int64_t tok = wk.token(grp);
        if constexpr (STATS) token_sumsq<C>(r, wave_sums, sumsq, tok, N, t, wk.slot, tm.last_ok);
        if (more) wait_vmem<0>();
        global_put<C, LAST, !C::kTwelve>(r, y + tok * C::kRow, tm.last_elem, tok < N && tm.last_ok);
    }
}

// One 16-byte vector per NV of a row, in the layout of phase PH, straight into registers (cached
// load).  Padding lanes of a 12 * 2^m row read the row's first block instead (in bounds) and hold zeros.
template <class C, int PH>
__device__ __forceinline__ void global_get(uint4 (&raw)[C::NV], const typename C::io::elem_t* row,
                                           unsigned thread_elem, bool ok) {
    const unsigned base = (!C::kTwelve || ok) ? thread_elem : 0u;
    static_for<0, C::NV>([&](auto c) {
        constexpr int Cc = decltype(c)::value;
        constexpr unsigned off = C::real(reg_elem_offset(C::plan.ph[PH], C::e, Cc * C::V));
        raw[Cc] = *reinterpret_cast<const uint4*>(row + base + off);
    });
    zero_padding<C>(raw, ok);
}

// forward for a few tokens (decoding, paper Sec. 5: one token per sequence and step): one token
// group per workgroup and nothing else.  With so little work a launch is one memory round trip
// long, so everything the group needs -- x, alpha, beta, the residual -- is requested at once,
// straight into registers, before anything is awaited; there is no token loop, no prefetch stage and
// no walk over the grid, whose set-up costs the persistent kernel about a microsecond per launch.
template <class C, bool RESID, bool STATS = false>
__global__ __launch_bounds__(C::BT) void forward_once_kernel(const typename C::io::elem_t* x,
                                                             const float* __restrict__ alpha,
                                                             const float* __restrict__ beta,
                                                             const typename C::io::elem_t* resid,
                                                             typename C::io::elem_t* y,
                                                             float* __restrict__ sumsq, int64_t N) {
    static_assert(!STATS || RESID, "the statistic belongs to the residual-stream output");
    __shared__ float wave_sums[STATS ? C::BT / 64 : 1];
    __shared__ __align__(16) float lds[C::kExchangeBytes / 4];
    constexpr int LAST = C::P - 1;
    const unsigned t = threadIdx.x % C::TPT, slot = threadIdx.x / C::TPT;
    ThreadMap<C> tm;
    tm.init(t, slot);
    const int64_t tok = (int64_t)blockIdx.x * C::G + slot;
    const int64_t row = tok < N ? tok : N - 1;                  // a ragged group re-reads the last token
    uint4 raw[C::NV], rraw[RESID ? C::NV : 1];
    global_get<C, 0>(raw, x + row * C::kRow, tm.first_elem, tm.first_ok);
    if constexpr (RESID) global_get<C, LAST>(rraw, resid + row * C::kRow, tm.last_elem, tm.last_ok);
    float a[C::E], b[C::E];
    param_get<C, LAST>(a, alpha, tm.last_elem, tm.last_ok, inv_sqrt_d<C>());
    param_get<C, LAST>(b, beta, tm.last_elem, tm.last_ok, 1.0f);
    HadamardB hb{}, hbp{};
    if constexpr (C::kMfma) hb = make_hadamard_b();
    if constexpr (C::kTwelve) hbp = make_paley_b(hb);
    const HadamardB& hb2 = C::kTwelve ? hbp : hb;
    float r[C::E];
    transform_from_raw<C, false>(r, raw, lds, tm, hb, hb2);
    if constexpr (RESID) {
        float res[C::E];
        unpack_all<C>(res, rraw);
#pragma unroll
        for (int i = 0; i < C::E; ++i) r[i] = res[i] + fmaf(r[i], a[i], b[i]);
    } else {
#pragma unroll
        for (int i = 0; i < C::E; ++i) r[i] = fmaf(r[i], a[i], b[i]);
    }
    if constexpr (STATS) token_sumsq<C>(r, wave_sums, sumsq, tok, N, t, slot, tm.last_ok);
    global_put<C, LAST, false>(r, y + tok * C::kRow, tm.last_elem, tok < N && tm.last_ok);
}

// backward:  z = H x (recomputed);  dalpha += dy z;  dbeta += dy;  dx = H_raw((alpha/sqrt d) dy)
// Each workgroup keeps its dalpha/dbeta sums in registers and at the end writes one row of partial
// sums; reduce_partials_kernel adds the rows in a fixed order, so the result does not depend on
// scheduling.
//
// Per iteration k (x(k) and dy(k) have landed in their stages):
//   raw <- stage X;  graw <- stage DY;  issue x(k+1), dy(k+1);  z = transform(raw);  sums;
//   g = alpha' dy;  transform back;  wait for everything pending;  store dx(k).
// As in the forward kernel the single wait precedes the stores and only covers loads issued a whole
// iteration earlier (and the previous token's stores).
//
// GRADS / DX select the outputs: without GRADS x is never read and no sums are kept (dx only, the
// traffic of a forward pass); without DX nothing is transformed back or stored.  With only one of
// the two, consecutive transforms run in the same order and need the trailing barrier again.
template <class C, bool GRADS, bool DX>
__global__ __launch_bounds__(C::BT) void backward_kernel(const typename C::io::elem_t* dy,
                                                         const typename C::io::elem_t* x,
                                                         const float* __restrict__ alpha,
                                                         typename C::io::elem_t* dx,
                                                         float* __restrict__ partials,   // [grid][2][kRow]
                                                         int64_t N) {
    static_assert(GRADS || DX, "nothing to compute");
    __shared__ __align__(16) float lds[C::kExchangeBytes / 4];
    __shared__ __align__(16) unsigned char stage_x_buf[GRADS ? C::kStageBytes : 16];
    __shared__ __align__(16) unsigned char stage_g_buf[C::kStageBytes];
    constexpr int LAST = C::P - 1;
    constexpr bool BOTH = GRADS && DX;
    const unsigned t = threadIdx.x % C::TPT;
    Walker<C> wk{N, (N + C::G - 1) / C::G, threadIdx.x / C::TPT};
    ThreadMap<C> tm;
    tm.init(t, wk.slot);
    HadamardB hb{}, hbp{};
    if constexpr (C::kMfma) hb = make_hadamard_b();
    if constexpr (C::kTwelve) hbp = make_paley_b(hb);
    const HadamardB& hb2 = C::kTwelve ? hbp : hb;
    unsigned char* stage_x = stage_x_buf + (GRADS ? (threadIdx.x >> 6) * (C::NV * 1024) : 0);
    unsigned char* stage_g = stage_g_buf + (threadIdx.x >> 6) * (C::NV * 1024);

    const int64_t step = gridDim.x;
    int64_t grp = blockIdx.x;
    if (grp < wk.groups) {
        if constexpr (GRADS) stage_issue<C, 0>(stage_x, x + wk.row(grp) * C::kRow, tm.first_elem, tm.first_ok);
        stage_issue<C, LAST>(stage_g, dy + wk.row(grp) * C::kRow, tm.last_elem, tm.last_ok);
    }

    float a[DX ? C::E : 1], da[GRADS ? C::E : 1], db[GRADS ? C::E : 1];
    if constexpr (DX) param_get<C, LAST>(a, alpha, tm.last_elem, tm.last_ok, inv_sqrt_d<C>());
    if constexpr (GRADS) {
#pragma unroll
        for (int i = 0; i < C::E; ++i) { da[i] = 0.0f; db[i] = 0.0f; }
    }
    wait_vmem<0>();
    for (; grp < wk.groups; grp += step) {
        const bool more = grp + step < wk.groups;
        uint4 raw[GRADS ? C::NV : 1], graw[C::NV];
        if constexpr (GRADS) {
            stage_read<C>(raw, stage_x);
            zero_padding<C>(raw, tm.first_ok);
        }
        stage_read<C>(graw, stage_g);
        zero_padding<C>(graw, tm.last_ok);
        if (more) {
            if constexpr (GRADS)
                stage_issue<C, 0>(stage_x, x + wk.row(grp + step) * C::kRow, tm.first_elem, tm.first_ok);
            stage_issue<C, LAST>(stage_g, dy + wk.row(grp + step) * C::kRow, tm.last_elem, tm.last_ok);
        }
        float g[C::E];
        const int64_t tok = wk.token(grp);
        const bool active = C::G == 1 || tok < N;             // one slot per workgroup: never ragged
        auto take_dy = [&]() {
            unpack_all<C>(g, graw);
            if constexpr (C::G > 1) {
                if (!active) {                                // ragged last group: contribute nothing
#pragma unroll
                    for (int i = 0; i < C::E; ++i) g[i] = 0.0f;
                }
            }
        };
        if constexpr (GRADS) {
            float r[C::E];
            transform_from_raw<C, !BOTH>(r, raw, lds, tm, hb, hb2);   // r = H_raw x, last layout
            take_dy();
#pragma unroll
            for (int i = 0; i < C::E; ++i) {
                da[i] = fmaf(g[i], r[i], da[i]);              // 1/sqrt d applied once at the end
                db[i] += g[i];
            }
        } else {
            take_dy();
        }
        if constexpr (DX) {
#pragma unroll
            for (int i = 0; i < C::E; ++i) g[i] *= a[i];
            transform_back<C, !BOTH>(g, lds, tm, hb, hb2);    // g = H_raw(alpha' dy), first layout
            if (more) wait_vmem<0>();
            global_put<C, 0, !C::kTwelve>(g, dx + tok * C::kRow, tm.first_elem, active && tm.first_ok);
        } else {
            if (more) wait_vmem<0>();
        }
    }
    if constexpr (GRADS) {
    // Sum the G token slots of this workgroup through LDS, then write the workgroup's row.
    if constexpr (C::G > 1) __syncthreads();      // the last exchange's reads are done everywhere
    const float s = inv_sqrt_d<C>();
    float* row = partials + (size_t)blockIdx.x * 2 * C::kRow;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        if constexpr (C::G == 1) {
            static_for<0, C::E / 4>([&](auto i) {
                constexpr int I = decltype(i)::value * 4;
                constexpr unsigned off = C::real(reg_elem_offset(C::plan.ph[LAST], C::e, I));
                const float4 q = which == 0 ? make_float4(da[I] * s, da[I + 1] * s, da[I + 2] * s, da[I + 3] * s)
                                            : make_float4(db[I], db[I + 1], db[I + 2], db[I + 3]);
                if (!C::kTwelve || tm.last_ok)
                    *reinterpret_cast<float4*>(row + which * C::kRow + tm.last_elem + off) = q;
            });
        } else {
            if (which == 0) lds_put<C, LAST>(da, lds + tm.lds_off[LAST]);
            else            lds_put<C, LAST>(db, lds + tm.lds_off[LAST]);
            __syncthreads();
            for (unsigned j = threadIdx.x; j < (unsigned)C::D; j += C::BT) {
                float acc = 0.0f;
#pragma unroll
                for (int gslot = 0; gslot < C::G; ++gslot) acc += lds[gslot * C::kTokenWords + C::phys(j)];
                if (C::valid(j)) row[which * C::kRow + C::real(j)] = which == 0 ? acc * s : acc;
            }
            __syncthreads();
        }
    }
    }   // GRADS
}

// One team's per-thread sums (last layout) -> the workgroup's row out[kRow], times `scale`.  With
// several token slots per workgroup the slots are added through `lds_sum` (an idle region of
// G * kTokenWords floats), between two workgroup barriers that every wave of the workgroup passes.
template <class C>
__device__ __forceinline__ void write_partial_row(const float (&acc)[C::E], float* lds_sum, float* out,
                                                  float scale, unsigned tid, const ThreadMap<C>& tm) {
    constexpr int LAST = C::P - 1;
    if constexpr (C::G == 1) {
        static_for<0, C::E / 4>([&](auto i) {
            constexpr int I = decltype(i)::value * 4;
            constexpr unsigned off = C::real(reg_elem_offset(C::plan.ph[LAST], C::e, I));
            const float4 q = make_float4(acc[I] * scale, acc[I + 1] * scale, acc[I + 2] * scale, acc[I + 3] * scale);
            if (!C::kTwelve || tm.last_ok) *reinterpret_cast<float4*>(out + tm.last_elem + off) = q;
        });
    } else {
        lds_put<C, LAST>(acc, lds_sum + tm.lds_off[LAST]);
        __syncthreads();
        for (unsigned j = tid; j < (unsigned)C::D; j += C::BT) {
            float sum = 0.0f;
#pragma unroll
            for (int gslot = 0; gslot < C::G; ++gslot) sum += lds_sum[gslot * C::kTokenWords + C::phys(j)];
            if (C::valid(j)) out[C::real(j)] = sum * scale;
        }
        __syncthreads();
    }
}

// backward (all three outputs) on three teams of waves per workgroup, 3 * C::BT threads, for the
// schedules with one LDS exchange per transform.  Wave w of every team holds the same elements of
// the token, so each SIMD runs one wave of each team and their matrix-core, vector and LDS phases
// overlap; one workgroup per CU keeps one token group per CU in flight.
//   X  waves: z = H_raw x (recomputed) and the dalpha sums
//   Y1 waves: fetch dy, the dbeta sums, alpha' dy, the stages before the exchange
//   Y2 waves: the stages after the exchange, the matrix-core rounds, store dx -- one token group
//             behind the other two teams
// Every wave passes two barriers per token group k, B1(k) and B2(k):
//   X (k) : [wait x(k); raw <- stage X; issue x(k+1); rounds; register stage; put X]  B1(k)
//           [get X; last stages; graw <- stage DY[k%2]; sums]                         B2(k)
//   Y1(k) : [wait dy(k); graw <- stage DY[k%2]; issue dy(k+1) -> DY[(k+1)%2]; sums; alpha'; stages]  B1(k)
//           [put Y]                                                                   B2(k)
//   Y2(k) : [get Y of group k-1; register stage; round 1]  B1(k)  [round 2; store dx(k-1)]  B2(k)
// and Y2 finishes the last group after the last barrier.  What the barriers order:
//   exchange region X: put before B1(k), get between B1(k) and B2(k), next put after B2(k);
//   exchange region Y: put between B1(k) and B2(k), get between B2(k) and B1(k+1);
//   stage DY[k%2]: filled by the Y1 waves' own loads (awaited before B1(k)), read by the X waves
//   between B1(k) and B2(k), refilled with dy(k+2) after B2(k).
// All teams run the same number of iterations, so they pass the same number of barriers.
// dx(k) is stored after x(k) and dy(k) have been read in full, so dx may alias either exactly.
template <class C>
__global__ __launch_bounds__(3 * C::BT) void backward_teams_kernel(const typename C::io::elem_t* dy,
                                                                   const typename C::io::elem_t* x,
                                                                   const float* __restrict__ alpha,
                                                                   typename C::io::elem_t* dx,
                                                                   float* __restrict__ partials,   // [grid][2][kRow]
                                                                   int64_t N) {
    static_assert(3 * C::BT <= 1024, "three teams must fit one workgroup");
    static_assert(C::kMfma && C::P == 2, "one exchange per transform");
    __shared__ __align__(16) float lds_x[C::kExchangeBytes / 4];
    __shared__ __align__(16) float lds_g[C::kExchangeBytes / 4];
    __shared__ __align__(16) unsigned char stage_x_buf[C::kStageBytes];
    __shared__ __align__(16) unsigned char stage_g_buf[2][C::kStageBytes];
    constexpr int LAST = 1;
    const unsigned team = threadIdx.x / C::BT;                // wave-uniform: BT is a multiple of 64
    const unsigned tid = threadIdx.x % C::BT;
    const unsigned t = tid % C::TPT;
    Walker<C> wk{N, (N + C::G - 1) / C::G, tid / C::TPT};
    ThreadMap<C> tm;
    tm.init(t, wk.slot);
    const unsigned wave_off = (tid >> 6) * (C::NV * 1024);
    unsigned char* stage_x = stage_x_buf + wave_off;
    unsigned char* stage_g0 = stage_g_buf[0] + wave_off;
    unsigned char* stage_g1 = stage_g_buf[1] + wave_off;

    const int64_t step = gridDim.x;
    int64_t grp = blockIdx.x;

    if (team == 0) {
        HadamardB hb{}, hbp{};
        hb = make_hadamard_b();
        if constexpr (C::kTwelve) hbp = make_paley_b(hb);
        const HadamardB& hb2 = C::kTwelve ? hbp : hb;
        if (grp < wk.groups) stage_issue<C, 0>(stage_x, x + wk.row(grp) * C::kRow, tm.first_elem, tm.first_ok);
        float da[C::E];
#pragma unroll
        for (int i = 0; i < C::E; ++i) da[i] = 0.0f;
        for (int par = 0; grp < wk.groups; grp += step, par ^= 1) {
            const bool more = grp + step < wk.groups;
            uint4 raw[C::NV], graw[C::NV];
            wait_vmem<0>();                                     // x(k) has landed
            stage_read<C>(raw, stage_x);
            zero_padding<C>(raw, tm.first_ok);
            if (more) stage_issue<C, 0>(stage_x, x + wk.row(grp + step) * C::kRow, tm.first_elem, tm.first_ok);
            const int64_t tok = wk.token(grp);
            const bool active = C::G == 1 || tok < N;
            float r[C::E], g[C::E];
            mfma_rounds_from_bf16<C>(r, raw, hb, hb2);
            run_stages<C, 0>(r);
            lds_put<C, 0>(r, lds_x + tm.lds_off[0]);
            exchange_barrier();                                 // B1(k)
            lds_get<C, LAST>(r, lds_x + tm.lds_off[LAST]);
            stage_read<C, false>(graw, par ? stage_g1 : stage_g0);     // fetched by the Y1 waves, read by both
            zero_padding<C>(graw, tm.last_ok);
            run_stages<C, LAST>(r);
            unpack_all<C>(g, graw);
            if constexpr (C::G > 1) {
                if (!active) {
#pragma unroll
                    for (int i = 0; i < C::E; ++i) g[i] = 0.0f;
                }
            }
#pragma unroll
            for (int i = 0; i < C::E; ++i) da[i] = fmaf(g[i], r[i], da[i]);
            exchange_barrier();                                 // B2(k)
        }
        write_partial_row<C>(da, lds_x, partials + (size_t)blockIdx.x * 2 * C::kRow, inv_sqrt_d<C>(), tid, tm);
    } else if (team == 1) {
        if (grp < wk.groups) stage_issue<C, LAST>(stage_g0, dy + wk.row(grp) * C::kRow, tm.last_elem, tm.last_ok);
        float a[C::E], db[C::E];
        param_get<C, LAST>(a, alpha, tm.last_elem, tm.last_ok, inv_sqrt_d<C>());
#pragma unroll
        for (int i = 0; i < C::E; ++i) db[i] = 0.0f;
        for (int par = 0; grp < wk.groups; grp += step, par ^= 1) {
            const bool more = grp + step < wk.groups;
            uint4 graw[C::NV];
            wait_vmem<0>();                                     // dy(k) has landed
            stage_read<C, false>(graw, par ? stage_g1 : stage_g0);
            zero_padding<C>(graw, tm.last_ok);
            if (more) stage_issue<C, LAST>(par ? stage_g0 : stage_g1, dy + wk.row(grp + step) * C::kRow, tm.last_elem, tm.last_ok);
            float g[C::E];
            unpack_all<C>(g, graw);
            if (C::G == 1 || wk.token(grp) < N) {               // a ragged last group's clamped rows add nothing
#pragma unroll
                for (int i = 0; i < C::E; ++i) db[i] += g[i];
            }
#pragma unroll
            for (int i = 0; i < C::E; ++i) g[i] *= a[i];
            run_stages<C, LAST>(g);
            exchange_barrier();                                 // B1(k): the Y2 waves have read token k-1
            lds_put<C, LAST>(g, lds_g + tm.lds_off[LAST]);
            exchange_barrier();                                 // B2(k)
        }
        // the stage buffers are idle now (same size as an exchange region)
        write_partial_row<C>(db, reinterpret_cast<float*>(&stage_g_buf[0][0]),
                             partials + (size_t)blockIdx.x * 2 * C::kRow + C::kRow, 1.0f, tid, tm);
    } else {
        HadamardB hb{}, hbp{};
        hb = make_hadamard_b();
        if constexpr (C::kTwelve) hbp = make_paley_b(hb);
        const HadamardB& hb2 = C::kTwelve ? hbp : hb;
        int64_t prev = -1;                                      // token group whose Y data is in the exchange region
        auto first_half = [&](float (&g)[C::E], f32x16 (&d1)[C::T]) {
            lds_get<C, 0>(g, lds_g + tm.lds_off[0]);
            run_stages<C, 0>(g);
            static_for<0, C::T>([&](auto tile) {
                constexpr int Tl = decltype(tile)::value;
                d1[Tl] = hadamard_round_f32(&g[16 * Tl], hb);
            });
        };
        auto second_half = [&](float (&g)[C::E], f32x16 (&d1)[C::T], int64_t grp_done) {
            static_for<0, C::T>([&](auto tile) {
                constexpr int Tl = decltype(tile)::value;
                float v[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = d1[Tl][i];
                const f32x16 d2 = hadamard_round_f32(v, hb2);
#pragma unroll
                for (int i = 0; i < 16; ++i) g[16 * Tl + i] = d2[i];
            });
            const int64_t tok = wk.token(grp_done);
            const bool active = C::G == 1 || tok < N;
            global_put<C, 0, !C::kTwelve>(g, dx + tok * C::kRow, tm.first_elem, active && tm.first_ok);
        };
        for (; grp < wk.groups; grp += step) {
            float g[C::E];
            f32x16 d1[C::T];
            if (prev >= 0) first_half(g, d1);
            exchange_barrier();                                 // B1(k)
            if (prev >= 0) second_half(g, d1, prev);
            exchange_barrier();                                 // B2(k): token k is in the exchange region
            prev = grp;
        }
        if (prev >= 0) {
            float g[C::E];
            f32x16 d1[C::T];
            first_half(g, d1);
            second_half(g, d1, prev);
        }
        if constexpr (C::G > 1) { __syncthreads(); __syncthreads(); }   // the other teams' closing barriers
    }
}

// out[which][j] = sum over rows of partials[row][which][j].  Workgroup = CG float4 columns x
// (1024 / CG) row lanes: lane r adds rows r, r + lanes, ... in index order, then the lane sums are
// combined by a fixed binary tree -- one association, independent of scheduling, so the result is
// bit-reproducible.  CG = 16 (256 contiguous bytes per row) for large d; CG = 4 keeps the grid wide
// (d/16 x 2 workgroups) for small d, where this kernel is otherwise pure latency.
template <int CG>
__global__ __launch_bounds__(1024) void reduce_partials_kernel(const float* __restrict__ partials,
                                                               int rows, int d,
                                                               float* __restrict__ dalpha,
                                                               float* __restrict__ dbeta) {
    constexpr int LANES = 1024 / CG;
    __shared__ float4 part[LANES][CG];
    const int cg = threadIdx.x % CG, lane_row = threadIdx.x / CG;
    const int col = (blockIdx.x * CG + cg) * 4;           // first of this thread's 4 columns
    const int which = blockIdx.y;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col < d) {
        for (int r = lane_row; r < rows; r += LANES) {
            const float4 q = *reinterpret_cast<const float4*>(partials + ((size_t)r * 2 + which) * d + col);
            acc.x += q.x; acc.y += q.y; acc.z += q.z; acc.w += q.w;
        }
    }
    part[lane_row][cg] = acc;
    __syncthreads();
#pragma unroll
    for (int half = LANES / 2; half >= 1; half >>= 1) {
        if (lane_row < half) {
            const float4 q = part[lane_row + half][cg];
            acc.x += q.x; acc.y += q.y; acc.z += q.z; acc.w += q.w;
            part[lane_row][cg] = acc;
        }
        __syncthreads();
    }
    if (lane_row == 0 && col < d)
        *reinterpret_cast<float4*>((which == 0 ? dalpha : dbeta) + col) = acc;
}

__global__ void zero_kernel(float* a, float* b, int d) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < d) { a[i] = 0.0f; b[i] = 0.0f; }
}

}  // namespace wht
