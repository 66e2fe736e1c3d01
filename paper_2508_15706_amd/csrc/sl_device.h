// Wave64 helpers for the gfx950 kernels: ballots, cross-lane butterflies and
// the fixed-shape fp64 summation tree.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define SL_DEV __device__ __forceinline__

SL_DEV unsigned long long sl_ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// Number of set bits of `m` below this lane.
SL_DEV int sl_mbcnt(unsigned long long m)
{
    return __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
}

// Orders this wavefront's LDS accesses: the hardware executes one wave's LDS
// instructions in order, so only the compiler has to be kept from moving
// memory operations across this point.  (Waves of a block never share LDS
// data in these kernels, so no s_barrier is needed.)
SL_DEV void sl_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

typedef float sl_f4 __attribute__((ext_vector_type(4)));
// The same vector in memory that is only 4-byte aligned (rows of a matrix whose column
// count is not a multiple of 4): still one 16-byte access - global memory accesses need
// no more than dword alignment on this target - so every streaming access below goes
// through it and a full tile of any matrix takes the vector path.
typedef float sl_f4u __attribute__((ext_vector_type(4), aligned(4)));

// Streaming (non-temporal) 16-byte accesses for data that is touched once.
// The *_at forms take a wave-uniform base and a 32-bit byte offset, which the
// compiler turns into scalar-base + 32-bit vector-offset addressing (one VGPR
// per address instead of two).
SL_DEV sl_f4 sl_load_stream(const float *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const sl_f4 *>(p));
}
SL_DEV void sl_store_stream(float *p, sl_f4 v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<sl_f4 *>(p));
}

// (`row_off` is a wave-uniform byte offset and goes into the scalar base, so
// that all accesses of a chunk share the single vector offset `lane_off`.)
SL_DEV sl_f4 sl_load_stream_at(const float *base, unsigned row_off, unsigned lane_off)
{
    const char *row = reinterpret_cast<const char *>(base) + row_off;
    return __builtin_nontemporal_load(reinterpret_cast<const sl_f4u *>(row + lane_off));
}
SL_DEV void sl_store_stream_at(float *base, unsigned row_off, unsigned lane_off, sl_f4 v)
{
    char *row = reinterpret_cast<char *>(base) + row_off;
    __builtin_nontemporal_store(v, reinterpret_cast<sl_f4u *>(row + lane_off));
}

// 16-byte streaming accesses at an address that is only 4-byte aligned.
SL_DEV sl_f4 sl_load_stream_u(const float *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const sl_f4u *>(p));
}
SL_DEV void sl_store_stream_u(float *p, sl_f4 v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<sl_f4u *>(p));
}

SL_DEV int sl_popc(unsigned long long m) { return __builtin_popcountll(m); }

SL_DEV int sl_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Cross-lane moves inside a row of 16 lanes as data-parallel-primitive modifiers (no trip
// through the LDS crossbar, unlike a shuffle).  With all 64 lanes active:
//   SL_DPP_XOR1, SL_DPP_XOR2  lane i reads lane i ^ 1, i ^ 2 (quad permutations);
//   SL_DPP_HALF_MIRROR        lane i reads lane 7 - i of its group of 8: a lane of the other quad;
//   SL_DPP_MIRROR             lane i reads lane 15 - i of its row: a lane of the other group of 8.
// In a butterfly whose earlier levels left the same value in every lane of a quad (a group of
// 8), the mirrors therefore deliver exactly what lane i ^ 4 (i ^ 8) would.
#define SL_DPP_XOR1 0xB1
#define SL_DPP_XOR2 0x4E
#define SL_DPP_HALF_MIRROR 0x141
#define SL_DPP_MIRROR 0x140
template <int CTRL>
SL_DEV int sl_dpp(int v) { return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false); }
template <int CTRL>
SL_DEV double sl_dpp(double v)
{
    return __hiloint2double(sl_dpp<CTRL>(__double2hiint(v)), sl_dpp<CTRL>(__double2loint(v)));
}
template <int CTRL>
SL_DEV unsigned long long sl_dpp(unsigned long long v)
{
    const unsigned lo = (unsigned)sl_dpp<CTRL>((int)(unsigned)v), hi = (unsigned)sl_dpp<CTRL>((int)(unsigned)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}
// Level l (0..5) of a butterfly over the wave: the value of the partner lane.
template <class T>
SL_DEV T sl_partner(T v, int l)
{
    switch (l) {
    case 0: return sl_dpp<SL_DPP_XOR1>(v);
    case 1: return sl_dpp<SL_DPP_XOR2>(v);
    case 2: return sl_dpp<SL_DPP_HALF_MIRROR>(v);
    case 3: return sl_dpp<SL_DPP_MIRROR>(v);
    default: return __shfl_xor(v, 1 << l);
    }
}

// (all 64 lanes active)
SL_DEV int sl_wave_max(int v)
{
#pragma unroll
    for (int l = 0; l < 4; ++l) v = max(v, sl_partner(v, l));       // every lane: its row's maximum
    return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

SL_DEV int sl_wave_min(int v)
{
#pragma unroll
    for (int l = 0; l < 4; ++l) v = min(v, sl_partner(v, l));
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

SL_DEV int sl_pow2ceil(int n)
{
    int p = 1;
    while (p < n) p <<= 1;
    return p;
}

// Adjacent-pair tree over the 64 lanes' values, `levels` levels (1 <= 2^levels
// <= 64): afterwards every lane whose index is a multiple of 2^levels holds the
// sum of its aligned group in the fixed pairing (v[2i] + v[2i+1] at each level).
// (All 64 lanes active.  a + b and b + a are the same double, so both lanes of a pair end
// up with the same sum, and after level l all 2^(l+1) lanes of a group hold the group's.)
SL_DEV double sl_wave_tree(double v, int levels)
{
#pragma unroll
    for (int l = 0; l < 6; ++l)
        if (l < levels) v = v + sl_partner(v, l);
    return v;
}

SL_DEV double sl_lane0(double v)
{
    int lo = __builtin_amdgcn_readfirstlane(__double2loint(v));
    int hi = __builtin_amdgcn_readfirstlane(__double2hiint(v));
    return __hiloint2double(hi, lo);
}

SL_DEV double sl_lane(double v, int l)
{
    int lo = __builtin_amdgcn_readlane(__double2loint(v), l);
    int hi = __builtin_amdgcn_readlane(__double2hiint(v), l);
    return __hiloint2double(hi, lo);
}

// sl_wave_tree's result in lane 0, as a wave-uniform value.  The four levels inside a row of
// 16 lanes leave each row's sum in every lane of the row; the two levels above them pair rows
// (0, 1), (2, 3) and then the pairs, read lane by lane instead of being shuffled.
SL_DEV double sl_wave_tree0(double v, int levels)
{
    v = sl_wave_tree(v, min(levels, 4));
    if (levels <= 4) return sl_lane0(v);
    const double r01 = sl_lane(v, 0) + sl_lane(v, 16);
    if (levels == 5) return r01;
    return r01 + (sl_lane(v, 32) + sl_lane(v, 48));
}

// Adjacent-pair trees of x and x*x over the E consecutive floats at v (E a power of two, v
// aligned for the widest read used); entries from index n on count as +0.0 and are not read
// (n a multiple of 4, or of 2 when E = 2: a read never straddles n).
template <int E>
SL_DEV void sl_lane_trees(const float *v, int n, double &sx, double &sxx)
{
    if constexpr (E == 2) {
        float2 q = make_float2(0.f, 0.f);
        if (n > 0) q = *reinterpret_cast<const float2 *>(v);
        const double x0 = q.x, x1 = q.y;
        sx = x0 + x1;
        sxx = x0 * x0 + x1 * x1;
    } else if constexpr (E == 4) {
        float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
        if (n > 0) q = *reinterpret_cast<const float4 *>(v);
        const double x0 = q.x, x1 = q.y, x2 = q.z, x3 = q.w;
        sx = (x0 + x1) + (x2 + x3);
        sxx = (x0 * x0 + x1 * x1) + (x2 * x2 + x3 * x3);
    } else {
        double a, aa, b, bb;
        sl_lane_trees<E / 2>(v, n, a, aa);
        sl_lane_trees<E / 2>(v + E / 2, n - E / 2, b, bb);
        sx = a + b;
        sxx = aa + bb;
    }
}

// Fixed summation trees of one chunk's k selected values x (canonical order, in LDS at
// `val`, 16-byte aligned; k a multiple of 4) and of their squares: the leaves of the
// two-level sums.  Each sequence is padded with +0.0 to P = pow2ceil(k) and reduced by adjacent
// pairs.  Lane l owns the P/64 consecutive entries from l*P/64 on - a subtree, summed in
// the lane - and one butterfly over the lanes finishes both trees.  MAXE bounds P/64 (the
// instantiation's largest k / 64, rounded up to a power of two).  The results are uniform.
template <int MAXE>
SL_DEV void sl_chunk_trees(int k, int lane, const float *val, double &sum_x, double &sum_xx)
{
    const int P = sl_pow2ceil(k);
    double x = 0.0, xx = 0.0;
    int levels = 6;
    if (P <= 64) {
        levels = 0;
        while ((1 << levels) < P) ++levels;
        x = lane < k ? (double)val[lane] : 0.0;
        xx = x * x;
    } else {
        const int E = P >> 6, n = k - lane * E;
        const float *v = val + lane * E;
        if (MAXE >= 2 && E == 2) sl_lane_trees<2>(v, n, x, xx);
        else if (MAXE >= 4 && E == 4) sl_lane_trees<4>(v, n, x, xx);
        else if (MAXE >= 8 && E == 8) sl_lane_trees<8>(v, n, x, xx);
        else if (MAXE >= 16 && E == 16) sl_lane_trees<16>(v, n, x, xx);
        else if (MAXE >= 32 && E == 32) sl_lane_trees<32>(v, n, x, xx);
        else if (MAXE >= 64 && E == 64) sl_lane_trees<64>(v, n, x, xx);
    }
    sum_x = sl_wave_tree0(x, levels);
    sum_xx = sl_wave_tree0(xx, levels);
}
