// Device-side building blocks shared by the kernels of the Tsetlin machine
// library: the counter-based random generator, wave64 helpers and the
// bit-sliced Tsetlin-automaton arithmetic.  gfx950 only (wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tsetlin {

// ---- random streams (counter word 0, bits 28..31) ----------------------
enum : uint32_t { STREAM_INIT = 0, STREAM_GATE = 1, STREAM_TYPE1 = 2, STREAM_NEGCLASS = 3 };

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
// as 1, 2, 3", SC'11).  The method needs one independent uniform per (seed,
// epoch, example, clause, literal); a counter-based generator gives that with
// no stored state: counter = (blk | stream<<28, clause, example lo,
// epoch | example hi<<24), key = seed.
struct U4 {
    uint32_t x, y, z, w;
};

// three-input bitwise functions in one instruction (gfx950 v_bitop3_b32; both
// truth tables are symmetric in their inputs)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return (uint32_t)__builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}
__device__ __forceinline__ uint32_t majority3(uint32_t a, uint32_t b, uint32_t c)
{
    return (uint32_t)__builtin_amdgcn_bitop3_b32(a, b, c, 0xE8);
}

// bit-select: where a bit of sel is 1 take it from b, else from c (operand truth
// tables 0xF0 / 0xCC / 0xAA, so sel ? b : c is 0xCA)
__device__ __forceinline__ uint32_t bitselect(uint32_t sel, uint32_t b, uint32_t c)
{
    return (uint32_t)__builtin_amdgcn_bitop3_b32(sel, b, c, 0xCA);
}

// One round costs two 32x32->64 multiplies (v_mad_u64_u32) and two 3-input xors.
__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return U4{c0, c1, c2, c3};
}

struct RngKey {
    uint32_t seed_lo, seed_hi;
};

__device__ __forceinline__ U4 draw(const RngKey &k, uint32_t stream, uint32_t blk, uint32_t g,
                                   uint64_t i, uint32_t epoch)
{
    return philox4x32_10(blk | (stream << 28), g, (uint32_t)i, epoch | ((uint32_t)(i >> 32) << 24),
                         k.seed_lo, k.seed_hi);
}

// ---- wave64 helpers ------------------------------------------------------
__device__ __forceinline__ uint64_t ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
__device__ __forceinline__ uint32_t readlane(uint32_t v, int l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, l);
}
// Orders the LDS traffic of one wavefront (writes by some lanes, then reads by
// others of the same wavefront) without involving the rest of the workgroup:
// the LDS executes a wavefront's instructions in order, so only the compiler
// has to be kept from reordering them.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int lane_id() { return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// ---- bit-sliced Tsetlin automata -------------------------------------------
// The 2N-state counter of 32 automata is held as 8 bit planes p[0..7] (plane b
// = bit b of every counter).  The stored value is (state - 1) + (128 - N), so
// plane 7 is exactly the Include decision (state > N) for every N <= 128 and
// the legal range is [128 - N, 127 + N].  Reinforcing Include adds 1,
// reinforcing Exclude subtracts 1 (Section 2.2 of the paper: the state is a
// counter), both saturating at the ends of the range.

// The planes of one register slot travel as one 8-wide vector value, so that a
// clause with many slots is a short array of vectors the compiler keeps in VGPRs.
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ void get_slot(const u32x8 &v, uint32_t (&s)[8])
{
#pragma unroll
    for (int b = 0; b < 8; ++b) s[b] = v[b];
}
__device__ __forceinline__ void put_slot(u32x8 &v, const uint32_t (&s)[8])
{
    u32x8 t;
#pragma unroll
    for (int b = 0; b < 8; ++b) t[b] = s[b];
    v = t;
}

struct SatConst {
    uint32_t kmax[8]; // per plane: 0 if that bit of the top value is 1, else ~0
    uint32_t kmin[8]; // same for the bottom value
};

template <bool FULL>
__device__ __forceinline__ uint32_t at_value(const uint32_t (&p)[8], const uint32_t (&k)[8], bool top)
{
    uint32_t eq = ~0u;
    if (FULL) { // range is 0..255: top = all ones, bottom = all zeros
        uint32_t a = p[0], o = p[0];
#pragma unroll
        for (int b = 1; b < 8; ++b) {
            a &= p[b];
            o |= p[b];
        }
        return top ? a : ~o;
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) eq &= (p[b] ^ k[b]);
    return eq;
}

// +1 on the automata selected by m (caller guarantees none of them is at the top)
__device__ __forceinline__ void ripple_inc(uint32_t (&p)[8], uint32_t m)
{
    uint32_t carry = m;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const uint32_t t = p[b] & carry;
        p[b] ^= carry;
        carry = t;
    }
}

// +1 on the automata selected by up and -1 on those selected by dn in one pass (up and dn disjoint, none
// of the former at the top, none of the latter at the bottom).  d marks the automata whose carry or
// borrow is still travelling: a carry goes on where the plane bit is 1, a borrow where it is 0, i.e.
// where the bit equals the direction.  Two operations per plane for both directions together.
__device__ __forceinline__ void ripple_updown(uint32_t (&p)[8], uint32_t up, uint32_t dn)
{
    uint32_t d = up | dn;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const uint32_t t = (uint32_t)__builtin_amdgcn_bitop3_b32(d, p[b], up, 0x90); // d & ~(p ^ up)
        p[b] ^= d;
        d = t;
    }
}

// -1 on the automata selected by m (none of them at the bottom)
__device__ __forceinline__ void ripple_dec(uint32_t (&p)[8], uint32_t m)
{
    uint32_t borrow = m;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const uint32_t t = ~p[b] & borrow;
        p[b] ^= borrow;
        borrow = t;
    }
}

} // namespace tsetlin
