// The coded wire format ("SLRICE02") on the device: what a wavefront needs to write and to
// read one chunk of it.  (The paper's appendix "Compression of indices in Top-k" names its index
// coder - Rice coding - and the rates it reaches, not the format; this one is the library's.)
//
// A chunk's ascending index list idx_0 < ... < idx_(k-1) is coded as gaps g_0 = idx_0,
// g_i = idx_i - idx_(i-1) - 1, each split by the Rice parameter b = floor(log2(2839 / k)) into a
// quotient q_i = g_i >> b and a remainder of b bits.  The two halves are stored apart:
//   * remainders: k fields of b bits (LSB first) at the start of the chunk's FIXED RECORD, padded
//     to 4 bytes, followed there by the k value fields as they stand in a plain record;
//   * quotients: one BIT VECTOR per chunk, the unary codes back to back - q_i one-bits, then a
//     zero bit - so entry i ends at the vector's i-th zero bit, at position
//     z_i = i + q_0 + ... + q_i, and the vector has k + Q bits, Q = sum of the q_i.
// So idx_i = i + ((z_i - i) << b) + r_0 + ... + r_i: every entry follows from the position of its
// own zero bit and a prefix sum of remainders, and a wave decodes a chunk's entries side by side.
//
// Buffer: "SLRICE02", uint64 total bytes; per tensor a 16-byte aligned block [table header]
// [directory][fixed records] at offsets that follow from the tensor list alone; then the
// quotient section: per group of 16 consecutive chunks of a tensor one run of their bit vectors,
// back to back, zero-padded to a 4-byte word.  A directory entry = uint32 offset of the group's
// run (in words from the start of the section) + the 16 chunks' Q (1 byte each while the
// largest possible Q is below 256, else 2).
#pragma once
#include "sl_device.h"
#include "sl_internal.h"

typedef unsigned __attribute__((address_space(3))) *sl_lds_words;

// LDS word |= v, &= v (the lanes of a wave may hit one word together)
SL_DEV void sl_lds_or(unsigned *p, unsigned v)
{
    __hip_atomic_fetch_or((sl_lds_words)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}
SL_DEV void sl_lds_and(unsigned *p, unsigned v)
{
    __hip_atomic_fetch_and((sl_lds_words)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}

// Lane i reads lane i - S of its row of 16 lanes, 0 where there is none (S = 1, 2, 4, 8).
template <int S>
SL_DEV int sl_row_shr(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x110 + S, 0xF, 0xF, true); }

// Inclusive prefix sum over the 64 lanes (all active): four steps inside each row of 16 lanes,
// then the totals of the rows below are added (read from the rows' last lanes).
SL_DEV int sl_wave_iscan(int v)
{
    v += sl_row_shr<1>(v);
    v += sl_row_shr<2>(v);
    v += sl_row_shr<4>(v);
    v += sl_row_shr<8>(v);
    const int t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31),
              t2 = __builtin_amdgcn_readlane(v, 47);
    const int row = (int)(threadIdx.x & 63) >> 4;
    return v + (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
}

// Value of lane `src` (any lane; all lanes call this together).
SL_DEV int sl_lane_read(int v, int src) { return __builtin_amdgcn_ds_bpermute(4 * src, v); }

// ---------------------------------------------------------------------------------- writer
// Codes the k ascending indices idx[0..k) (LDS) of one chunk.  uv (LDS, G.ua words) receives
// the bit vector, bits beyond its k + Q left as ones; rw (LDS, G.rem_bytes / 4 words) the
// remainder fields, padding zero.  Returns Q (uniform).  Called by all 64 lanes; the caller
// orders its own earlier LDS accesses before the call and reads uv / rw after it.
// Indices that are not strictly ascending (a malformed plain record - a compressor never
// produces one) are coded as gap 0, and a vector that would outgrow k + qmax bits is cut there.
SL_DEV int sl_coded_emit(const SlCodedGeom &G, int lane, const unsigned short *idx, unsigned *uv, unsigned *rw)
{
    const int k = G.k, b = G.b, nrw = G.rem_bytes >> 2;
    for (int w = lane; w < G.ua; w += 64) uv[w] = 0xFFFFFFFFu;
    for (int w = lane; w < nrw; w += 64) rw[w] = 0u;
    sl_wave_sync();
    const int limit = k + G.qmax;            // bits of the longest vector
    // A lane owns ceil(k / 64) CONSECUTIVE entries: one wave scan for the whole chunk, and the lanes of one
    // store instruction are that many entries apart, so that at high densities they land in different
    // words of the vector (64 neighbouring entries would share two or three words, and the LDS atomics on
    // one word take turns).
    const int E = (k + 63) >> 6, m0 = lane * E, m1 = min(k, m0 + E);
    const int first_prev = (m0 > 0 && m0 < k) ? (int)idx[m0 - 1] : -1;
    int prev = first_prev, qsum = 0;
    for (int m = m0; m < m1; ++m) {
        const int cur = (int)idx[m];
        qsum += max(cur - prev - 1, 0) >> b;
        prev = cur;
    }
    const int incl = sl_wave_iscan(qsum);
    int qrun = incl - qsum;                  // quotients of all entries before the lane's first
    prev = first_prev;
    for (int m = m0; m < m1; ++m) {
        const int cur = (int)idx[m];
        const int gap = max(cur - prev - 1, 0);
        prev = cur;
        qrun += gap >> b;
        const unsigned r = (unsigned)gap & ((1u << b) - 1u);
        const int z = qrun + m;              // position of entry m's zero bit
        if (z < limit) sl_lds_and(&uv[z >> 5], ~(1u << (z & 31)));
        if (b) {
            const int bit = m * b, sh = bit & 31;
            sl_lds_or(&rw[bit >> 5], r << sh);
            if (sh + b > 32) sl_lds_or(&rw[(bit >> 5) + 1], r >> (32 - sh));
        }
    }
    const int carry = __builtin_amdgcn_readlane(incl, 63);
    sl_wave_sync();
    return min(carry, G.qmax);
}

// ---------------------------------------------------------------------------------- reader
// One directory entry (16-byte loads need only 4-byte alignment): for the chunk at position
// `pos` of its group, the word offset of the group's run, the bit at which the chunk's vector
// starts inside the run and the vector's length.  Quotient sums are clamped to qmax, so that
// a malformed entry still describes a vector of at most k + qmax bits that starts below
// 15 (k + qmax).
struct SlVecPlace {
    unsigned run_word;      // the group's run, in words from the start of the quotient section
    int start_bit;          // first bit of the chunk's vector inside the run
    int nbits;              // k + Q
};

// pointers into global memory, for addresses that are put together from integers (a generic
// pointer would turn every access into a flat load that LDS waits have to sit out)
typedef const unsigned char __attribute__((address_space(1))) *sl_gbytes;
typedef const unsigned __attribute__((address_space(1))) *sl_gwords;
typedef unsigned sl_u4u __attribute__((ext_vector_type(4), aligned(4)));
typedef const sl_u4u __attribute__((address_space(1))) *sl_gu4;

// The words of a directory entry as loaded (the loads are issued here; nothing waits for them
// until sl_coded_dir_parse reads the words).
struct SlDirWords {
    unsigned run_word;
    sl_u4u lo, hi;          // the 16 quotient sums: 16 bytes, or 32 when they are two bytes each
};

SL_DEV SlDirWords sl_coded_dir_load(const SlCodedGeom &G, sl_gbytes entry)
{
    SlDirWords W;
    const sl_gwords e = reinterpret_cast<sl_gwords>(entry);
    W.run_word = e[0];
    W.lo = *reinterpret_cast<sl_gu4>(e + 1);
    W.hi = sl_u4u{0u, 0u, 0u, 0u};
    if (G.qf == 2) W.hi = *reinterpret_cast<sl_gu4>(e + 5);
    return W;
}

// Field j (0..15) of a directory entry's quotient sums, j a compile-time constant.
template <int J>
SL_DEV unsigned sl_dir_field(int qf, sl_u4u lo, sl_u4u hi)
{
    if (qf == 2) {
        const sl_u4u v = J < 8 ? lo : hi;
        const unsigned w = ((J >> 1) & 3) == 0 ? v.x : ((J >> 1) & 3) == 1 ? v.y : ((J >> 1) & 3) == 2 ? v.z : v.w;
        return (w >> (16 * (J & 1))) & 0xFFFFu;
    }
    const unsigned w = (J >> 2) == 0 ? lo.x : (J >> 2) == 1 ? lo.y : (J >> 2) == 2 ? lo.z : lo.w;
    return (w >> (8 * (J & 3))) & 0xFFu;
}

template <int J>
SL_DEV void sl_dir_sum(int qf, int qmax, sl_u4u lo, sl_u4u hi, int pos, int &before, int &own)
{
    if constexpr (J < SL_RICE_GROUP) {
        const int qc = min((int)sl_dir_field<J>(qf, lo, hi), qmax);
        before += J < pos ? qc : 0;
        own = J == pos ? qc : own;
        sl_dir_sum<J + 1>(qf, qmax, lo, hi, pos, before, own);
    }
}

SL_DEV SlVecPlace sl_coded_dir_parse(const SlCodedGeom &G, unsigned run_word, sl_u4u lo, sl_u4u hi, int pos)
{
    SlVecPlace P;
    P.run_word = run_word;
    int before = 0, own = 0;
    sl_dir_sum<0>(G.qf, G.qmax, lo, hi, pos, before, own);
    P.start_bit = pos * G.k + before;
    P.nbits = G.k + own;
    return P;
}

SL_DEV SlVecPlace sl_coded_dir_entry(const SlCodedGeom &G, sl_gbytes entry, int pos)
{
    const SlDirWords W = sl_coded_dir_load(G, entry);
    return sl_coded_dir_parse(G, W.run_word, W.lo, W.hi, pos);
}
