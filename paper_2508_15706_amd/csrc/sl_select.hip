// Kernel A of sl_compress: error-feedback accumulate fused with the chunk-wise
// Top-k selection (Eq. (2) line 1 and the Top-k of line 2; Section 3.3 last
// paragraph for the chunking).
//
// One 64-lane wavefront owns one 4096-element chunk, 64 elements per lane in
// registers; a workgroup is several independent waves on adjacent chunks (so
// that a workgroup streams 1 KB of every matrix row it touches).  HBM traffic
// per chunk: 16 KB of e and 16 KB of delta read once, 16 KB of e written once
// (all as streaming 16-byte accesses), plus 3k/2 bytes of packed indices,
// 4k bytes of selected values and 16 bytes of partial sums.
//
// Register r = 4*i + cc of lane l holds local index j = 256*i + 4*l + cc, i.e.
// the lane's i-th 16-byte load.  With rows of 64 elements this is row
// 4*i + l/16, columns 4*(l%16) .. +3 for both chunk layouts.
//
// Selection = exact k-th largest magnitude key T (key = bit pattern of |a|)
// by bitwise bisection with wave ballots as the counting primitive, made cheap
// by pruning first:
//   1. every lane keeps the maxima of GPL interleaved groups of its registers;
//      the k-th largest of those 64*GPL maxima is a lower bound L of T (there
//      are k distinct elements >= L);
//   2. one ordered compaction over the registers moves the entries with key
//      >= L (about 1.4k of them when 64*GPL = 2k) into LDS in ascending local
//      index;
//   3. T is bisected over that short list, and a second compaction over the
//      list emits the selected entries, still in ascending local index; ties
//      at T go to the lowest indices.
// Partial chunks, a candidate list that overflows (massive ties) and k > 512
// take the general route: T bisected over the registers directly and one
// ordered compaction over the registers - slower, same result.
#include "sl_coded.h"

namespace {

// LDS candidate list of the pruned route, entries of 8 bytes: 512, or 1024 with 16 groups per lane
constexpr int cand_cap(int gpl) { return gpl == 16 ? 1024 : 512; }

#ifndef SL_SELECT_BOUND_BITS
#define SL_SELECT_BOUND_BITS 12   // bits of the pruning bound that are decided (0 = all)
#endif
#ifndef SL_SELECT_PFE8
#define SL_SELECT_PFE8 4
#endif

struct SelectArgs {
    const SlChunkDesc *desc;
    float *e;
    const float *delta;             // the pseudo-gradient, or theta_outer when theta_local is set
    const float *theta_local;       // non-null: delta = theta_outer - theta_local, formed on the fly
    const unsigned char *pending;   // payload whose values are still to be subtracted from e
    float beta;
    int frozen;
    int k;
    int bits, hdr_bytes, rec_bytes; // value width of the payloads and the sizes that follow from it
    unsigned seed_hash;     // Random-k: fmix32(seed), see random_key
    int lds_per_wave;
    int pend_off;           // offset of the pending-correction tables in a wave's LDS
    int pend_words;         // the pending record is staged in LDS as whole words (large k), see pend_half
    float *vals;            // [n_chunks * k] selected values, canonical order
    double *leafA;          // [2][n_chunks] per-chunk tree sums of x and x*x
    unsigned char *payload;
    long long n_chunks;
    // coded wire format written next to the plain record (null: not wanted): the remainder fields go
    // to their place in the buffer, the chunk's quotient bit vector and quotient sum to the workspace
    unsigned char *coded;
    const SlTensorDev *tensors;
    SlCodedGeom G;
    unsigned *uvec;
    unsigned short *qsum;
};

SL_DEV int key_of(float x) { return (int)(__float_as_uint(x) & 0x7FFFFFFFu); }

// Random-k (the paper's ablation "Random-k vs. Top-k"): every position gets a
// pseudo-random 31-bit key from a counter-based generator built on the 32-bit
// finalizer of MurmurHash3 (Appleby, public domain),
//     key = fmix32(fmix32(fmix32(seed) ^ chunk) ^ j) >> 1,
// chunk = index of the chunk in the list, j = local index; the k largest keys
// are selected by the same machinery as the k largest magnitudes.
SL_DEV unsigned fmix32(unsigned h)
{
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}

// Largest T in [lo, hi] with count_ge(T) >= k, given count_ge(lo) >= k and
// 0 <= lo <= hi.  All values are wave-uniform.
// With `steps` > 0 only that many bits below the highest one in which lo and hi differ are
// decided and the rest left zero: a value that is not above the exact answer and still has
// count_ge >= k.
template <class CountGE>
SL_DEV int bisect_kth(int lo, int hi, int k, CountGE count_ge, int steps = 0)
{
    if (lo >= hi) return lo;
    const int top = 31 - __clz(lo ^ hi);
    const int last = steps > 0 ? max(0, top - steps + 1) : 0;
    int T = hi & ~(int)((2u << top) - 1u);
    for (int b = top; b >= last; --b) {
        const int cand = T | (1 << b);
        if (count_ge(cand) >= k) T = cand;
    }
    return T;
}

// General route.  key[r] is the magnitude key of register r, or -1 for a
// position outside the tensor; sg0/sg1 hold the sign of register r at bit
// 31 - (r & 31) of sg[r / 32].  Writes the k selected (value, index) pairs in
// ascending local index to sel_val / sel_idx.
//
// The threshold T (the k-th largest key) is found in two stages.  A pass over all 64 registers
// of every lane is the expensive unit, so only the leading SL_SELECT_COARSE_BITS bits of T are
// bisected that way; this leaves T inside a bucket [T1, T1 + width) that holds few keys (about
// fifty at a quarter density on Gaussian data).  One more pass copies the bucket's keys to
// `list` (LDS, SL_SELECT_LIST_CAP ints, any order) and counts the keys above the bucket; the
// remaining bits are bisected over the list alone.  A bucket that does not fit the list (many
// equal keys) is bisected over the registers as before.
#ifndef SL_SELECT_COARSE_BITS
#define SL_SELECT_COARSE_BITS 12
#endif
#define SL_SELECT_LIST_CAP 512
template <bool VALUES_FROM_A>
SL_DEV void select_general(int (&key)[64], const float (&a)[64], unsigned sg0, unsigned sg1, int k, int lane,
                           float *sel_val, unsigned short *sel_idx, int *list)
{
    auto count_regs = [&](int x) {
        int n = 0;
#pragma unroll
        for (int r = 0; r < 64; ++r) n += sl_popc(sl_ballot(key[r] >= x));
        return n;
    };
    int lmax = key[0];
#pragma unroll
    for (int r = 1; r < 64; ++r) lmax = max(lmax, key[r]);
    const int hi = sl_wave_max(lmax);
    int T = 0, n_ge = 0, n_gt = -1;         // n_gt: keys above T, where the list already gave it
    const int top = hi > 0 ? 31 - __clz(hi) : 0;
    const int last = top - SL_SELECT_COARSE_BITS + 1;    // lowest bit the coarse stage decides
    if (last >= 3) {
        // T1: the leading bits of T.  count(T1) >= k, and count(T1 + width) < k: T1 + width is either
        // beyond every key or a value the bisection tried and rejected.
        const int T1 = bisect_kth(0, hi, k, count_regs, SL_SELECT_COARSE_BITS);
        const int width = 1 << last, upper = T1 | (width - 1);
        int n_above = 0, m = 0;
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            // (a position outside the tensor has key -1: never above, and far outside the bucket)
            const bool in = (unsigned)(key[r] - T1) < (unsigned)width;
            const unsigned long long mb = sl_ballot(in);
            n_above += sl_popc(sl_ballot(key[r] > upper));
            if (mb) {
                const int pos = m + sl_mbcnt(mb);
                if (in && pos < SL_SELECT_LIST_CAP) list[pos] = key[r];
                m += sl_popc(mb);
            }
        }
        sl_wave_sync();
        if (m <= SL_SELECT_LIST_CAP) {
            constexpr int SLOTS = SL_SELECT_LIST_CAP / 64;
            const int nslots = (m + 63) >> 6;
            int ck[SLOTS];
#pragma unroll
            for (int s = 0; s < SLOTS; ++s) {
                const int p = s * 64 + lane;
                ck[s] = (s < nslots && p < m) ? list[p] : -1;
            }
            auto count_list = [&](int x) {
                int n = 0;
#pragma unroll
                for (int s = 0; s < SLOTS; ++s)
                    if (s < nslots) n += sl_popc(sl_ballot(ck[s] >= x));
                return n;
            };
            // the (k - n_above)-th largest key of the bucket
            T = bisect_kth(T1, upper, k - n_above, count_list);
            n_ge = n_above + count_list(T);
            n_gt = n_above + (T == upper ? 0 : count_list(T + 1));    // keys above T: beyond the bucket, or in it
        } else {
            T = bisect_kth(T1, upper, k, count_regs);
            n_ge = count_regs(T);
        }
        sl_wave_sync();                     // the list shares LDS with nothing live, but keep its reads
                                            // ahead of whatever the caller stores next
    } else {
        T = bisect_kth(0, hi, k, count_regs);
        n_ge = count_regs(T);
    }
    const bool ties = n_ge != k;            // more keys equal to T than slots left
    int need = 0;                           // tie entries to take, lowest indices first
    if (ties) {
        if (n_gt < 0) {
            n_gt = 0;
#pragma unroll
            for (int r = 0; r < 64; ++r) n_gt += sl_popc(sl_ballot(key[r] > T));
        }
        need = k - n_gt;
    }
    int base = 0, tbase = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        bool f[4];
        if (!ties) {
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) f[cc] = key[4 * i + cc] >= T;
        } else {
            // rank of a tie entry among all tie entries in ascending local index
            bool eq[4];
            int trank = tbase, tcnt = 0;
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                eq[cc] = key[4 * i + cc] == T;
                const unsigned long long m = sl_ballot(eq[cc]);
                trank += sl_mbcnt(m);
                tcnt += sl_popc(m);
            }
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                f[cc] = key[4 * i + cc] > T || (eq[cc] && trank < need);
                trank += eq[cc] ? 1 : 0;
            }
            tbase += tcnt;
        }
        int pos = base, cnt = 0;
        unsigned long long any = 0;
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const unsigned long long m = sl_ballot(f[cc]);
            pos += sl_mbcnt(m);
            cnt += sl_popc(m);
            any |= m;
        }
        if (any) {
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const int r = 4 * i + cc;
                if (f[cc] && pos < k) {
                    const unsigned sg = r < 32 ? sg0 : sg1;
                    const unsigned sign = (sg << (r & 31)) & 0x80000000u;
                    // a magnitude key and the sign give the value back; a random key does not
                    sel_val[pos] = VALUES_FROM_A ? a[r] : __uint_as_float((unsigned)key[r] | sign);
                    sel_idx[pos] = (unsigned short)(256 * i + 4 * lane + cc);
                    ++pos;
                }
            }
        }
        base += cnt;
    }
}

// 3 waves per SIMD (<= 168 VGPRs): measured faster than 2 (no spills) or 4 (heavy spills).
#ifndef SL_SELECT_WAVES_PER_EU
#define SL_SELECT_WAVES_PER_EU 3
#endif
#define SL_SELECT_BOUNDS __launch_bounds__(256, SL_SELECT_WAVES_PER_EU)

// MODE 0: a = beta*e + delta.  MODE 1 (PARAMS): the pseudo-gradient is formed on
// the fly from two parameter arenas (a separate instantiation, so that the plain
// path keeps its register budget).  MODE 2 (SUBK): no accumulate at all - the
// buffer itself is the operand of Top-k and its selected entries are set to
// zero, m <- m - Top-k(m) (Section 3.2, DiLoCo-LOM-Sub-k); nothing else is written.
// TWO_BIT: payloads carry 2-bit codes (the paper's setting; the width is then a
// compile-time constant); otherwise the width is A.bits.
// RANDOM: Random-k instead of Top-k (only with GPL = 0: random keys cannot be pruned by magnitude).
template <int GPL, int MODE, bool TWO_BIT, bool RANDOM = false>
__global__ void SL_SELECT_BOUNDS k_select(SelectArgs A)
{
    constexpr bool PARAMS = MODE == 1, SUBK = MODE == 2;
    static_assert(!RANDOM || GPL == 0, "Random-k takes the general route");
    extern __shared__ __align__(16) unsigned char smem_all[];
    const int lane = threadIdx.x & 63;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= A.n_chunks) return;
    unsigned char *smem = smem_all + (size_t)wave * A.lds_per_wave;
    const SlChunkDesc d = A.desc[c];
    const int k = A.k;

    // LDS of this wave: [candidates 8*CAND_CAP][sel_val 4k][sel_idx 2k]
    uint2 *cand = reinterpret_cast<uint2 *>(smem);
    constexpr int CAND_CAP = cand_cap(GPL), CAND_SLOTS = CAND_CAP / 64;
    // (the general route's key list takes the place of the candidates: 2 KB when GPL = 0)
    const size_t cand_bytes = GPL > 0 ? sizeof(uint2) * CAND_CAP : sizeof(int) * SL_SELECT_LIST_CAP;
    float *sel_val = reinterpret_cast<float *>(smem + cand_bytes);
    unsigned short *sel_idx = reinterpret_cast<unsigned short *>(smem + cand_bytes + 4 * (size_t)k);

    float *ec = A.e + d.base;
    const float *dc = SUBK ? nullptr : A.delta + d.base;
    const int lr = lane >> 4, lc = (lane & 15) * 4;
    const unsigned stride = (unsigned)d.stride;
    const bool full = d.flags & SLC_FULL;

    float a[64];
    unsigned long long inside = ~0ull;      // bit r: register r is a position of the tensor
    bool done = false;

    // Pending error update of the previous round (deferred residual): the values its
    // record transmits are subtracted from e as e is read, see pend_half.
    float *corr = nullptr;                  // pending values of one half of the chunk, by position
    float *lutl = nullptr;                  // centroid table of the widths that keep it in LDS
    const bool pend = A.pending != nullptr;
    const int bits = TWO_BIT ? 2 : A.bits;
    const unsigned char *prec = nullptr, *pcodes = nullptr;
    float4 plut = make_float4(0.f, 0.f, 0.f, 0.f);
    float p_lutv = 0.f;                     // other widths: table entry `lane`, parked in LDS later
    // record entries per lane that are fetched early: all of them up to k = 256
    constexpr int PFE = GPL == 8 ? SL_SELECT_PFE8 : 2;
    unsigned p_w[PFE], p_c[PFE];
    // k > 256 only: a record of whole words that is a multiple of eight entries is
    // staged in LDS and decoded eight entries per lane, instead of entry by entry from global memory.
    constexpr bool BIG = GPL == 0 || GPL == 16;     // the instantiations that serve k > 256
    constexpr int PW = GPL == 16 ? 4 : BIG ? 8 : 1;   // words per lane fetched early: 1 KB (k <= 512), 2 KB
    unsigned pw[PW];
    const bool pwords = BIG && pend && A.pend_words;
    const int rec_words = (TWO_BIT ? 7 * k / 4 : A.rec_bytes) >> 2;
    unsigned *stg = nullptr;
    // The bytes of the value field of entry m: the code's byte window, or the fp32 value.
    auto value_window = [&](int m) -> unsigned {
        if (bits == 32) return reinterpret_cast<const unsigned *>(pcodes)[m];
        const int bit = m * bits;
        unsigned w = pcodes[bit >> 3];
        if ((bit & 7) + bits > 8) w |= (unsigned)pcodes[(bit >> 3) + 1] << 8;
        return w;
    };
    if (pend) {
        corr = reinterpret_cast<float *>(smem + A.pend_off);
        lutl = corr + SL_CHUNK / 2;
        prec = A.pending + d.rec_off;
        pcodes = prec + 3 * k / 2;
        const unsigned char *lutg =
            A.pending + (TWO_BIT ? sl_lut_off(d, 16, 7 * k / 4) : sl_lut_off(d, A.hdr_bytes, A.rec_bytes));
        if (bits == 2) plut = *reinterpret_cast<const float4 *>(lutg);
        else if (bits != 32 && lane < (1 << bits)) p_lutv = reinterpret_cast<const float *>(lutg)[lane];
        if (pwords) {
            // large records (general route): the first 2 KB as whole words, coalesced
            stg = reinterpret_cast<unsigned *>(lutl + 16);
#pragma unroll
            for (int u = 0; u < PW; ++u) {
                const int w = lane + 64 * u;
                pw[u] = w < rec_words ? reinterpret_cast<const unsigned *>(prec)[w] : 0u;
            }
        } else {
#pragma unroll
            for (int u = 0; u < PFE; ++u) {
                const int m = lane + 64 * u;
                p_w[u] = p_c[u] = 0;
                if (m < k) {
                    const int b0 = (3 * m) >> 1;
                    p_w[u] = (unsigned)prec[b0] | ((unsigned)prec[b0 + 1] << 8);
                    p_c[u] = value_window(m);
                }
            }
        }
    }
    // The pending values of half h of the chunk (local indices h*2048 ..) as a dense array
    // in LDS, +0.0f where nothing is pending: the error update is then e - corr, position by
    // position (x - (+0.0f) leaves every x as it is, signed zeros included), with one 16-byte LDS
    // read per 16-byte access of e and no look-ups.  A record's positions are distinct, so its
    // entries are plain stores.  Called with the chunk's bulk loads in flight.
    auto pend_half = [&](int h) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
            reinterpret_cast<float4 *>(corr)[64 * u + lane] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (h == 0) {
            if (bits != 2 && bits != 32 && lane < (1 << bits)) lutl[lane] = p_lutv;
            if constexpr (BIG) {
                if (pwords) {
#pragma unroll
                    for (int u = 0; u < PW; ++u) {
                        const int w = lane + 64 * u;
                        if (w < rec_words) stg[w] = pw[u];
                    }
                    for (int w = lane + 64 * PW; w < rec_words; w += 64)       // beyond the early words
                        stg[w] = reinterpret_cast<const unsigned *>(prec)[w];
                }
            }
        }
        sl_wave_sync();
        auto put = [&](unsigned j, float q) {
            if ((int)(j >> 11) == h) corr[j & (SL_CHUNK / 2 - 1)] = q;
        };
        const float pl0 = plut.x, pl1 = plut.y, pl2 = plut.z, pl3 = plut.w;
        auto value_of = [&](unsigned field) -> float {       // field: the entry's code in the low bits
            if (bits == 2) {      // two selects on the code's bits, on four scalars: selects between the
                                  // elements of a vector become an indexed read of a copy in private memory
                const float lo = (field & 1u) ? pl1 : pl0, hi = (field & 1u) ? pl3 : pl2;
                return (field & 2u) ? hi : lo;
            }
            return lutl[field & ((1u << bits) - 1u)];
        };
        if (pwords) {
            if constexpr (BIG) {
                const unsigned char *scodes = reinterpret_cast<const unsigned char *>(stg) + 3 * k / 2;
                for (int o = lane; o < (k >> 3); o += 64) {
                    // entries 8o .. 8o+7: three words of indices, `bits` bytes of codes
                    const unsigned w0 = stg[3 * o], w1 = stg[3 * o + 1], w2 = stg[3 * o + 2];
                    unsigned cw = 0;
                    if (bits != 32)
                        for (int b = 0; b < bits; ++b) cw |= (unsigned)scodes[o * bits + b] << (8 * b);
                    // (written out entry by entry: an array of the eight indices ends up in private memory)
                    auto put_e = [&](int e, unsigned j) __attribute__((always_inline)) {
                        put(j, bits == 32 ? reinterpret_cast<const float *>(scodes)[8 * o + e]
                                          : value_of(cw >> (e * bits)));
                    };
                    put_e(0, w0 & 0xFFFu);
                    put_e(1, (w0 >> 12) & 0xFFFu);
                    put_e(2, (w0 >> 24) | ((w1 & 0xFu) << 8));
                    put_e(3, (w1 >> 4) & 0xFFFu);
                    put_e(4, (w1 >> 16) & 0xFFFu);
                    put_e(5, (w1 >> 28) | ((w2 & 0xFFu) << 4));
                    put_e(6, (w2 >> 8) & 0xFFFu);
                    put_e(7, w2 >> 20);
                }
            }
        } else {
            auto entry = [&](int m, unsigned w, unsigned vw) {
                const unsigned j = (m & 1) ? (w >> 4) : (w & 0xFFFu);
                put(j, bits == 32 ? __uint_as_float(vw) : value_of(vw >> ((m * bits) & 7)));
            };
#pragma unroll
            for (int u = 0; u < PFE; ++u)
                if (lane + 64 * u < k) entry(lane + 64 * u, p_w[u], p_c[u]);
            for (int m = lane + 64 * PFE; m < k; m += 64) {
                const int b0 = (3 * m) >> 1;
                entry(m, (unsigned)prec[b0] | ((unsigned)prec[b0 + 1] << 8), value_window(m));
            }
        }
        sl_wave_sync();
    };
    // e - corr for 16-byte access i of this lane (local indices 256*i + 4*lane ..)
    auto pend_sub = [&](sl_f4 ee, int i) -> sl_f4 {
        const float4 cq = reinterpret_cast<const float4 *>(corr)[64 * (i & 7) + lane];
        ee.x = ee.x - cq.x, ee.y = ee.y - cq.y, ee.z = ee.z - cq.z, ee.w = ee.w - cq.w;
        return ee;
    };

    if (full) {
        // ------------------------------------------------------------ a = beta*e + delta
        const unsigned o0 = 4u * (lr * stride + lc);   // byte offset of this lane's first load
        const unsigned step = 16u * stride;            // four rows further, in bytes
        sl_f4 ev[16], dv[16];
        if constexpr (SUBK) {
#pragma unroll
            for (int i = 0; i < 16; ++i) ev[i] = sl_load_stream_at(ec, i * step, o0);
        } else if constexpr (PARAMS) {
            // pseudo-gradient delta = theta_outer - theta_local (one fp32 subtraction).
            // Three input streams: the chunk is taken in four quarters (four 16-byte
            // accesses per lane and stream each), finished one after the other, so that
            // only a quarter of each stream sits in registers next to the result.
            const float *lc_ = A.theta_local + d.base;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                sl_f4 dq[4], tq[4], eq[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) dq[u] = sl_load_stream_at(dc, (4 * q + u) * step, o0);
#pragma unroll
                for (int u = 0; u < 4; ++u) tq[u] = sl_load_stream_at(lc_, (4 * q + u) * step, o0);
                if (!A.frozen) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) eq[u] = sl_load_stream_at(ec, (4 * q + u) * step, o0);
                }
                if (pend && (q & 1) == 0) pend_half(q >> 1);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = 4 * q + u;
                    const sl_f4 g = dq[u] - tq[u];
                    sl_f4 v = g;
                    if (!A.frozen) {
                        sl_f4 ee = eq[u];
                        if (pend) ee = pend_sub(ee, i);
                        v.x = fmaf(A.beta, ee.x, g.x);
                        v.y = fmaf(A.beta, ee.y, g.y);
                        v.z = fmaf(A.beta, ee.z, g.z);
                        v.w = fmaf(A.beta, ee.w, g.w);
                        sl_store_stream_at(ec, i * step, o0, v);
                    }
                    a[4 * i + 0] = v.x, a[4 * i + 1] = v.y, a[4 * i + 2] = v.z, a[4 * i + 3] = v.w;
                }
                __builtin_amdgcn_sched_barrier(0);   // keep the quarters apart: no hoisting of the next loads
            }
        } else {
            if (!A.frozen) {
#pragma unroll
                for (int i = 0; i < 16; ++i) ev[i] = sl_load_stream_at(ec, i * step, o0);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) dv[i] = sl_load_stream_at(dc, i * step, o0);
        }
        if (!SUBK && !PARAMS && pend) pend_half(0);   // (half 1 follows inside the loop below, once half 0 is used up)
#pragma unroll
        for (int i = 0; i < (PARAMS ? 0 : 16); ++i) {
            sl_f4 v;
            if constexpr (SUBK) {
                v = ev[i];
            } else if (!A.frozen) {
                if (pend) {
                    if (i == 8) pend_half(1);
                    ev[i] = pend_sub(ev[i], i);
                }
                v.x = fmaf(A.beta, ev[i].x, dv[i].x);
                v.y = fmaf(A.beta, ev[i].y, dv[i].y);
                v.z = fmaf(A.beta, ev[i].z, dv[i].z);
                v.w = fmaf(A.beta, ev[i].w, dv[i].w);
                sl_store_stream_at(ec, i * step, o0, v);
            } else {
                v = dv[i];
            }
            a[4 * i + 0] = v.x, a[4 * i + 1] = v.y, a[4 * i + 2] = v.z, a[4 * i + 3] = v.w;
        }

    } else {
        // ------------------------------------------------------------ partial chunk
        // A lane whose four columns of a row all lie inside the tensor still moves them
        // with one 16-byte access; a lane that straddles the edge goes element by element.
        // As for a full chunk, every load is issued before the first result is needed.
        const int rows = d.rows, cols = d.cols, last_cols = d.last_cols;
        const bool need_e = SUBK || !A.frozen;
        auto limit_of = [&](int i) -> int {            // columns of this lane's row 4*i + lr that exist
            const int row = 4 * i + lr;
            return row < rows - 1 ? cols : (row == rows - 1 ? last_cols : 0);
        };
        // (in two halves of 32 rows, as much as the registers hold next to the results)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            sl_f4 pe[8], pd[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = 8 * h + u, lim = limit_of(i);
                const unsigned o0 = (4 * i + lr) * stride + lc;
                pe[u] = pd[u] = sl_f4{0.f, 0.f, 0.f, 0.f};
                if (lc + 3 < lim) {
                    if (need_e) pe[u] = sl_load_stream_u(ec + o0);
                    if constexpr (!SUBK) {
                        pd[u] = sl_load_stream_u(dc + o0);
                        if constexpr (PARAMS) pd[u] = pd[u] - sl_load_stream_u(A.theta_local + d.base + o0);
                    }
                } else {
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) {
                        if (lc + cc < lim) {
                            if (need_e) pe[u][cc] = ec[o0 + cc];
                            if constexpr (!SUBK)
                                pd[u][cc] = PARAMS ? dc[o0 + cc] - (A.theta_local + d.base)[o0 + cc] : dc[o0 + cc];
                        }
                    }
                }
            }
            if constexpr (!SUBK) {
                if (pend) pend_half(h);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = 8 * h + u, lim = limit_of(i);
                const unsigned o0 = (4 * i + lr) * stride + lc;
                sl_f4 vout;
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    float v = 0.0f;
                    if (lc + cc < lim) {
                        if constexpr (SUBK) {
                            v = pe[u][cc];
                        } else if (!A.frozen) {
                            float ee = pe[u][cc];
                            if (pend) ee = ee - corr[256 * u + 4 * lane + cc];
                            v = fmaf(A.beta, ee, pd[u][cc]);
                        } else {
                            v = pd[u][cc];
                        }
                    } else {
                        inside &= ~(1ull << (4 * i + cc));
                    }
                    vout[cc] = v;
                    a[4 * i + cc] = v;
                }
                if (!SUBK && !A.frozen) {
                    if (lc + 3 < lim) {
                        sl_store_stream_u(ec + o0, vout);
                    } else {
#pragma unroll
                        for (int cc = 0; cc < 4; ++cc)
                            if (lc + cc < lim) ec[o0 + cc] = vout[cc];
                    }
                }
            }
        }
    }

    // Pruned selection.  A partial chunk takes it too: its positions outside the tensor hold 0.0f,
    // i.e. key 0, and can only enter the candidate list if the bound L is 0 - then the list
    // overflows (it would hold all 4096 positions) and the general route, which knows the
    // outside positions, takes over.
    if constexpr (GPL > 0) {
        constexpr int G = GPL;
        // group g of a lane = its registers r with r % G == g
        int gm[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            int m = key_of(a[g]);
#pragma unroll
            for (int r = g + G; r < 64; r += G) m = max(m, key_of(a[r]));
            gm[g] = m;
        }
        int lmin = gm[0], lmax = gm[0];
#pragma unroll
        for (int g = 1; g < G; ++g) lmin = min(lmin, gm[g]), lmax = max(lmax, gm[g]);
        const int hi = sl_wave_max(lmax);               // largest key of the chunk
        const int lo = sl_wave_min(lmin);
        // L = k-th largest group maximum, or a little less: a lower bound of T, because k
        // distinct elements are >= L (64*G >= k groups).  A bound is all that is needed, so
        // only its leading bits are decided - a slightly longer candidate list for half the
        // counting passes.
        const int L = bisect_kth(lo, hi, k, [&](int x) {
            int n = 0;
#pragma unroll
            for (int g = 0; g < G; ++g) n += sl_popc(sl_ballot(gm[g] >= x));
            return n;
        }, SL_SELECT_BOUND_BITS);
        // ordered compaction of the entries with key >= L
        int ncand = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            bool f[4];
            int pos = ncand, cnt = 0;
            unsigned long long any = 0;
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                f[cc] = key_of(a[4 * i + cc]) >= L;
                const unsigned long long m = sl_ballot(f[cc]);
                pos += sl_mbcnt(m);
                cnt += sl_popc(m);
                any |= m;
            }
            if (any) {
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    if (f[cc]) {
                        if (pos < CAND_CAP)
                            cand[pos] = make_uint2(__float_as_uint(a[4 * i + cc]),
                                                   (unsigned)(256 * i + 4 * lane + cc));
                        ++pos;
                    }
                }
            }
            ncand += cnt;
        }
        sl_wave_sync();
        if (ncand <= CAND_CAP && (full || L > 0)) {
            const int nslots = (ncand + 63) >> 6;
            int ck[CAND_SLOTS];
#pragma unroll
            for (int s = 0; s < CAND_SLOTS; ++s) {
                const int p = s * 64 + lane;
                ck[s] = (s < nslots && p < ncand) ? (int)(cand[p].x & 0x7FFFFFFFu) : -1;
            }
            auto count_cand = [&](int x) {
                int n = 0;
#pragma unroll
                for (int s = 0; s < CAND_SLOTS; ++s)
                    if (s < nslots) n += sl_popc(sl_ballot(ck[s] >= x));
                return n;
            };
            const int T = bisect_kth(L, hi, k, count_cand);
            const int n_ge = count_cand(T);
            const bool ties = n_ge != k;
            int need = 0;
            if (ties) {
                int n_gt = 0;
#pragma unroll
                for (int s = 0; s < CAND_SLOTS; ++s)
                    if (s < nslots) n_gt += sl_popc(sl_ballot(ck[s] > T));
                need = k - n_gt;
            }
            int base = 0, tbase = 0;
#pragma unroll
            for (int s = 0; s < CAND_SLOTS; ++s) {
                if (s < nslots) {
                    bool f;
                    if (!ties) {
                        f = ck[s] >= T;
                    } else {
                        const bool eq = ck[s] == T;
                        const unsigned long long me = sl_ballot(eq);
                        f = ck[s] > T || (eq && tbase + sl_mbcnt(me) < need);
                        tbase += sl_popc(me);
                    }
                    const unsigned long long m = sl_ballot(f);
                    const int pos = base + sl_mbcnt(m);
                    if (f && pos < k) {
                        const uint2 v = cand[s * 64 + lane];
                        sel_val[pos] = __uint_as_float(v.x);
                        sel_idx[pos] = (unsigned short)v.y;
                    }
                    base += sl_popc(m);
                }
            }
            done = true;
        }
    }

    if (!done) {
        int key[64];
        unsigned sg0 = 0, sg1 = 0;
        if (!RANDOM && full) {
#pragma unroll
            for (int r = 0; r < 64; ++r) key[r] = key_of(a[r]);
        } else {
#pragma unroll
            for (int r = 0; r < 64; ++r) {
                const bool outside = !((inside >> r) & 1ull);
                if constexpr (RANDOM) {
                    const unsigned j = 256u * (r >> 2) + 4u * lane + (r & 3);
                    key[r] = outside ? -1 : (int)(fmix32(fmix32(A.seed_hash ^ (unsigned)c) ^ j) >> 1);
                } else {
                    key[r] = outside ? -1 : key_of(a[r]);
                }
            }
        }
        // the signs, one bit per register (a position outside the tensor is never selected, so its
        // bit is never read): sg = (sg << 1) | sign, as one funnel shift
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            const unsigned u = __float_as_uint(a[r]);
            if (r < 32) sg0 = __builtin_amdgcn_alignbit(sg0, u, 31);
            else sg1 = __builtin_amdgcn_alignbit(sg1, u, 31);
        }
        select_general<RANDOM>(key, a, sg0, sg1, k, lane, sel_val, sel_idx, reinterpret_cast<int *>(smem));
    }
    sl_wave_sync();

    if constexpr (SUBK) {
        // m - Top-k(m): x - x = +0.0 at the selected positions, the rest stays as it is
        for (int p = lane; p < k; p += 64) {
            const unsigned j = sel_idx[p];
            ec[(j >> 6) * stride + (j & 63u)] = 0.0f;
        }
        return;
    }

    // ---------------------------------------------------------------- outputs
    unsigned char *rec = A.payload + d.rec_off;

    // the selected values, four LDS reads in flight per round of stores
    float *recv = bits == 32 ? reinterpret_cast<float *>(rec + 3 * k / 2) : nullptr;   // unquantized: the values
                                                              // themselves follow the indices (4-byte aligned)
    for (int p0 = lane; p0 < k; p0 += 256) {
        float t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = p0 + 64 * u < k ? sel_val[p0 + 64 * u] : 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (p0 + 64 * u < k) {
                A.vals[c * k + p0 + 64 * u] = t[u];
                if (recv) recv[p0 + 64 * u] = t[u];
            }
    }

    if ((k & 15) == 0) {
        // 12-bit index stream, one 32-bit word per lane (records are 4-byte aligned)
        unsigned *rw = reinterpret_cast<unsigned *>(rec);
        const int nwords = 3 * k / 8;
        for (int w = lane; w < nwords; w += 64) {
            const int bit0 = 32 * w;
            int m = bit0 / 12;
            unsigned word = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q, ++m) {
                const int sh = 12 * m - bit0;
                if (m < k && sh < 32) {
                    const unsigned v = sel_idx[m];
                    word |= sh >= 0 ? v << sh : v >> (-sh);
                }
            }
            rw[w] = word;
        }
    } else {
        const int nbytes = 3 * k / 2;
        for (int b = lane; b < nbytes; b += 64) {
            const int bit0 = 8 * b;
            const int m = bit0 / 12;
            const int sh = bit0 - 12 * m;             // 0, 4 or 8
            unsigned v = (unsigned)sel_idx[m] >> sh;
            if (sh == 8 && m + 1 < k) v |= (unsigned)sel_idx[m + 1] << 4;
            rec[b] = (unsigned char)v;
        }
    }

    // the coded form of the index list (the candidate list's LDS is free by now)
    if (A.coded) {
        const SlCodedGeom &G = A.G;
        const SlTensorDev td = A.tensors[d.tensor];
        unsigned *uv = reinterpret_cast<unsigned *>(smem), *rw = uv + G.ua;
        const int nrw = G.rem_bytes >> 2;
        const int Q = sl_coded_emit(G, lane, sel_idx, uv, rw);
        unsigned char *fix = A.coded + td.cfix_off + (long long)d.local_chunk * G.cfix;
        for (int w = lane; w < nrw; w += 64) reinterpret_cast<unsigned *>(fix)[w] = rw[w];
        if (bits == 32) {
            // unquantized: the values follow the remainders as they follow the indices of a plain record
            for (int m = lane; m < k; m += 64) reinterpret_cast<float *>(fix + G.rem_bytes)[m] = sel_val[m];
        } else if ((G.val_bytes & 3) && lane == 0) {
            // the record's last word holds value fields and padding: cleared here, the codes come later
            *reinterpret_cast<unsigned *>(fix + G.cfix - 4) = 0u;
        }
        unsigned *uvo = A.uvec + (size_t)c * G.ua;
        const int words = (k + Q + 31) >> 5;
        for (int w = lane; w < words; w += 64) uvo[w] = uv[w];
        if (lane == 0) A.qsum[c] = (unsigned short)Q;
    }

    // per-chunk leaves of the quantizer's mean / variance sums
    double s1, s2;
    constexpr int MAXE = GPL == 0 ? 64 : GPL <= 2 ? 1 : GPL / 2;      // pow2ceil(largest k served) / 64
    sl_chunk_trees<MAXE>(k, lane, sel_val, s1, s2);
    if (lane == 0) {
        A.leafA[c] = s1;
        A.leafA[A.n_chunks + c] = s2;
    }
}

}  // namespace

static unsigned host_fmix32(unsigned h)
{
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}

static int launch_select(const sl_plan *p, float *e, const float *delta, const float *theta_local, float beta,
                         int frozen, const unsigned char *pending, unsigned char *payload, unsigned char *coded,
                         unsigned char *ws, bool sub_only, bool random, unsigned seed, hipStream_t st)
{
    if (p->n_chunks == 0) return SL_OK;
    const int k = p->k;
    const bool pruned = k <= 512;
    SelectArgs A;
    A.desc = p->d_desc;
    A.e = e;
    A.delta = delta;
    A.theta_local = theta_local;
    A.pending = pending;
    A.beta = beta;
    A.frozen = frozen;
    A.k = k;
    A.bits = p->bits;
    A.hdr_bytes = p->hdr_bytes;
    A.rec_bytes = p->rec_bytes;
    A.seed_hash = host_fmix32(seed);
    {
        size_t b = pruned ? sizeof(uint2) * cand_cap(k > 256 ? 16 : 8) : sizeof(int) * SL_SELECT_LIST_CAP;
        // (the coded form's bit vector and remainder words reuse this first part: at most 128 + 64 words)
        b += (6 * (size_t)k + 7) & ~(size_t)7;
        b = (b + 15) & ~(size_t)15;
        // k > 256: a pending record of whole words and whole groups of eight entries is staged in LDS
        A.pend_words = pending && k > 256 && (p->rec_bytes & 3) == 0 && (k & 7) == 0 && p->rec_bytes <= 8192;
        // the pending tables are dead before the selection starts: they share its LDS
        A.pend_off = 0;
        if (pending) {
            const size_t pb = (SL_CHUNK / 2) * sizeof(float) + 16 * sizeof(float) +
                              (A.pend_words ? (size_t)p->rec_bytes : 0);
            if (b < pb) b = pb;
        }
        A.lds_per_wave = (int)((b + 15) & ~(size_t)15);
    }
    A.vals = sub_only ? nullptr : reinterpret_cast<float *>(ws + p->ws_vals);
    A.leafA = sub_only ? nullptr : reinterpret_cast<double *>(ws + p->ws_leafA);
    A.payload = payload;
    A.n_chunks = p->n_chunks;
    A.coded = sub_only ? nullptr : coded;
    A.tensors = p->d_tensors;
    A.G = p->cg;
    A.uvec = (sub_only || !coded) ? nullptr : reinterpret_cast<unsigned *>(ws + p->ws_uvec);
    A.qsum = (sub_only || !coded) ? nullptr : reinterpret_cast<unsigned short *>(ws + p->ws_qsum);
    // waves (= chunks) per workgroup: 4 adjacent chunks when their LDS fits
    const int wpb = 4 * (size_t)A.lds_per_wave <= 65536 ? 4 : 1;
    const dim3 grid((unsigned)((p->n_chunks + wpb - 1) / wpb)), block(64 * wpb);
    const size_t lds = (size_t)A.lds_per_wave * wpb;
#define SL_LAUNCH_SELECT(MODE, TWO)                                                                   \
    do {                                                                                              \
        if (k <= 32) hipLaunchKernelGGL((k_select<1, MODE, TWO>), grid, block, lds, st, A);         \
        else if (k <= 64) hipLaunchKernelGGL((k_select<2, MODE, TWO>), grid, block, lds, st, A);    \
        else if (k <= 128) hipLaunchKernelGGL((k_select<4, MODE, TWO>), grid, block, lds, st, A);   \
        else if (k <= 256) hipLaunchKernelGGL((k_select<8, MODE, TWO>), grid, block, lds, st, A);   \
        else if (k <= 512) hipLaunchKernelGGL((k_select<16, MODE, TWO>), grid, block, lds, st, A);  \
        else hipLaunchKernelGGL((k_select<0, MODE, TWO>), grid, block, lds, st, A);                 \
    } while (0)
    const bool two = p->bits == 2;
    if (sub_only) {
        SL_LAUNCH_SELECT(2, false);
    } else if (random) {
        if (two) hipLaunchKernelGGL((k_select<0, 0, true, true>), grid, block, lds, st, A);
        else hipLaunchKernelGGL((k_select<0, 0, false, true>), grid, block, lds, st, A);
    } else if (theta_local) {
        if (two) SL_LAUNCH_SELECT(1, true);
        else SL_LAUNCH_SELECT(1, false);
    } else {
        if (two) SL_LAUNCH_SELECT(0, true);
        else SL_LAUNCH_SELECT(0, false);
    }
#undef SL_LAUNCH_SELECT
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    return SL_OK;
}

int slk_select(const sl_plan *p, float *e, const float *delta, const float *theta_local, float beta,
               int frozen, const unsigned char *pending, unsigned char *payload, unsigned char *coded,
               unsigned char *ws, hipStream_t st)
{
    return launch_select(p, e, delta, theta_local, beta, frozen, pending, payload, coded, ws, false, false, 0u, st);
}

int slk_select_random(const sl_plan *p, float *e, const float *delta, float beta, int frozen,
                      const unsigned char *pending, unsigned char *payload, unsigned char *ws, unsigned seed,
                      hipStream_t st)
{
    return launch_select(p, e, delta, nullptr, beta, frozen, pending, payload, nullptr, ws, false, true, seed, st);
}

int slk_sub_topk(const sl_plan *p, float *m, hipStream_t st)
{
    return launch_select(p, m, nullptr, nullptr, 1.0f, 0, nullptr, nullptr, nullptr, nullptr, true, false, 0u, st);
}
