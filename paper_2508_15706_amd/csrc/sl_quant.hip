// Kernels B-E of sl_compress: the per-tensor 2-bit statistical quantizer
// (Section 4, experimental set-up) and the error-feedback residual (Eq. (2)
// line 2, Algorithm 1 error update).
//
//   B  per tensor: fixed-tree fp64 sums of x and x*x over its selected values
//      -> mean mu and variance;
//   C  per chunk: 2-bit codes from (x - mu)^2 vs T, codes packed into the
//      payload record, per-bin partial sums and counts;
//   D  per tensor: fixed-tree sums per bin -> centroid LUT, written as the
//      tensor block's header;
//   E  per chunk: e[idx] = a - LUT[code] at the k selected positions.
//
// Sums over a tensor are two-level: a tree over each chunk's k entries (the
// leaves, produced by kernels A and C) and a tree over the chunk leaves in
// chunk order.  Both trees pad with +0.0 to a power of two and add adjacent
// pairs, so the result does not depend on scheduling.
#include "sl_device.h"
#include "sl_internal.h"

namespace {

constexpr int RED_THREADS = 1024;
constexpr int RED_TILE = 4 * RED_THREADS;   // leaves reduced per block iteration

struct RedShared {
    double wsum[RED_THREADS / 64];
    double stack[40];
    double result;
    unsigned long long cnt[4];
};

// Adjacent-pair tree over leaf[0..n) padded with +0.0 (to a multiple of 4096 and
// then to a power of two; extra +0.0 leaves do not change a sum).  Called by all
// RED_THREADS threads of the block; returns the sum to every thread.
__device__ double block_tree_sum(const double *leaf, long long n, RedShared &sh)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long tiles = n > 0 ? (n + RED_TILE - 1) / RED_TILE : 1;
    long long pushed = 0;
    for (long long tile = 0; tile < tiles; ++tile) {
        const long long b = tile * RED_TILE + 4ll * tid;
        const double x0 = b + 0 < n ? leaf[b + 0] : 0.0;
        const double x1 = b + 1 < n ? leaf[b + 1] : 0.0;
        const double x2 = b + 2 < n ? leaf[b + 2] : 0.0;
        const double x3 = b + 3 < n ? leaf[b + 3] : 0.0;
        double v = (x0 + x1) + (x2 + x3);
        v = sl_wave_tree(v, 6);
        if (lane == 0) sh.wsum[wave] = v;
        __syncthreads();
        if (wave == 0) {
            double w = lane < RED_THREADS / 64 ? sh.wsum[lane] : 0.0;
            w = sl_wave_tree(w, 4);
            if (lane == 0) {
                // binary-counter stack: combines equal-sized aligned subtrees
                long long idx = pushed;
                int lvl = 0;
                while (idx & 1) {
                    w = sh.stack[lvl] + w;
                    idx >>= 1;
                    ++lvl;
                }
                sh.stack[lvl] = w;
            }
        }
        ++pushed;
        __syncthreads();
    }
    if (tid == 0) {
        long long P = 1;
        int top = 0;
        while (P < tiles) P <<= 1, ++top;
        for (; pushed < P; ++pushed) {          // +0.0 padding tiles
            double w = 0.0;
            long long idx = pushed;
            int lvl = 0;
            while (idx & 1) {
                w = sh.stack[lvl] + w;
                idx >>= 1;
                ++lvl;
            }
            sh.stack[lvl] = w;
        }
        sh.result = sh.stack[top];
    }
    __syncthreads();
    const double r = sh.result;
    __syncthreads();
    return r;
}

// ------------------------------------------------------------------ kernel B
__global__ void __launch_bounds__(RED_THREADS)
k_tensor_stats(const SlTensorDev *tensors, const double *leafA, long long n_chunks_total, int k,
               SlTensorStat *tstat)
{
    __shared__ RedShared sh;
    const SlTensorDev td = tensors[blockIdx.x];
    const double S1 = block_tree_sum(leafA + td.chunk0, td.n_chunks, sh);
    const double S2 = block_tree_sum(leafA + n_chunks_total + td.chunk0, td.n_chunks, sh);
    if (threadIdx.x == 0) {
        const double M = (double)(td.n_chunks * (long long)k);
        const double mu = S1 / M;
        const double q = S2 / M;
        const double p = mu * mu;
        double var = q - p;
        if (var < 0.0) var = 0.0;
        tstat[blockIdx.x].mu = mu;
        tstat[blockIdx.x].var = var;
    }
}

// ------------------------------------------------------------------ kernel C
struct CodeArgs {
    const SlChunkDesc *desc;
    const SlTensorStat *tstat;
    const float *vals;
    double *leafC;          // [4][n_chunks] per-chunk tree sums of the values of each bin
    unsigned *cnt;          // [4][n_chunks] entries per bin
    unsigned char *payload;
    long long n_chunks;
    int k;
    // coded wire format next to the plain record (null: not wanted): the value fields of a chunk are
    // the same bytes in both, in the coded buffer they follow the chunk's remainder fields
    unsigned char *coded;
    const SlTensorDev *tensors;
    int cfix, rem_bytes;
    int park;               // k_codes_b: the codes of the first pass are kept in LDS for the later ones
};

// Where a chunk's value fields go in the coded buffer (null when none is written).
SL_DEV unsigned char *coded_values(const CodeArgs &A, const SlChunkDesc &d)
{
    if (!A.coded) return nullptr;
    return A.coded + A.tensors[d.tensor].cfix_off + (long long)d.local_chunk * A.cfix + A.rem_bytes;
}

template <int LV>
struct BinStacksT {      // one binary-counter stack of partial tree sums per bin, LV levels (k <= 2^(LV-1))
    double a[LV], b[LV], c[LV], d[LV];
};
using BinStacks = BinStacksT<13>;

// Folds entry m (values v0..v3 for the four bins) into the stacks: while bit L
// of m is set the partial sum of level L is the left sibling and is added; the
// first clear bit is where the new partial sum is parked.
template <int L, int LV>
SL_DEV void stack_push(BinStacksT<LV> &s, int m, double v0, double v1, double v2, double v3)
{
    if constexpr (L < LV) {
        if ((m >> L) & 1) {
            stack_push<L + 1>(s, m, s.a[L] + v0, s.b[L] + v1, s.c[L] + v2, s.d[L] + v3);
        } else {
            s.a[L] = v0, s.b[L] = v1, s.c[L] = v2, s.d[L] = v3;
        }
    }
}

constexpr int CODE_WAVES = 2;        // waves per workgroup
#ifndef SL_CODES_WAVE_FROM
#define SL_CODES_WAVE_FROM 129        // k from which a wave, not a lane, owns a chunk in kernel C
#endif
// (... and at any k on a list of fewer chunks than the plan's codes_wave_below, 32768 unless set: with a lane per
// chunk such a list leaves most of the chip without a wave)

// One LANE per chunk, 64 consecutive chunks per wave.  The selected values of
// the 64 chunks are read with coalesced 16-byte loads, 64 entries per chunk at a
// time, and transposed through LDS so that every lane walks its own chunk's
// values in ascending index.  A lane then needs no cross-lane traffic at all:
// the code is two fp64 compares, and the per-bin fixed-tree sums are kept in a
// binary-counter stack (entry m is folded into the partial sums of the aligned
// subtrees that end at m, which reproduces the adjacent-pair tree exactly).
// The entry index is uniform over the wave, so the stack walk is scalar control flow.
// LV: levels of the stacks (k <= 2^(LV-1)); TC: entries per chunk that are transposed at a
// time.  Few levels and a small tile (the paper's densities: k <= 256) leave room for four
// waves per SIMD, which this latency- and VALU-bound kernel needs.
template <int LV, int TC, int WAVES_PER_EU>
__global__ void __launch_bounds__(64 * CODE_WAVES, WAVES_PER_EU) k_codes(CodeArgs A)
{
    constexpr int PITCH = TC + 1;            // conflict-free column reads
    __shared__ float tile_all[CODE_WAVES][64 * PITCH];
    const int lane = threadIdx.x & 63, k = A.k;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c0 = ((long long)blockIdx.x * CODE_WAVES + wave) * 64;
    if (c0 >= A.n_chunks) return;
    float *tile = tile_all[wave];
    const long long c = c0 + lane;
    const bool live = c < A.n_chunks;

    double mu = 0.0, T = 0.0;
    unsigned char *codes_out = nullptr, *codes_out2 = nullptr;
    if (live) {
        const SlChunkDesc d = A.desc[c];
        mu = A.tstat[d.tensor].mu;
        T = 9.0 * A.tstat[d.tensor].var;      // squared distance of the outer edges (3 sigma)
        codes_out = A.payload + d.rec_off + 3 * k / 2;
        codes_out2 = coded_values(A, d);
    }

    BinStacksT<LV> st;
#pragma unroll
    for (int l = 0; l < LV; ++l) st.a[l] = st.b[l] = st.c[l] = st.d[l] = 0.0;
    unsigned n_b[4] = {0u, 0u, 0u, 0u};
    unsigned word = 0;

    constexpr int LPR = TC / 4;              // lanes that load one row of the tile
    const int lr = lane / LPR, lc = (lane % LPR) * 4;
    for (int s0 = 0; s0 < k; s0 += TC) {
        const int ncol = min(TC, k - s0);          // multiple of 4
        sl_wave_sync();
#pragma unroll
        for (int i = 0; i < LPR; ++i) {
            const int row = (64 / LPR) * i + lr;
            if (c0 + row < A.n_chunks && lc < ncol) {
                const float4 v = *reinterpret_cast<const float4 *>(A.vals + (c0 + row) * k + s0 + lc);
                float *t = tile + row * PITCH + lc;
                t[0] = v.x, t[1] = v.y, t[2] = v.z, t[3] = v.w;
            }
        }
        sl_wave_sync();
        for (int col = 0; col < ncol; ++col) {
            const int m = s0 + col;
            const float xf = tile[lane * PITCH + col];
            const double x = (double)xf;
            const double dlt = x - mu;
            const double dd = dlt * dlt;
            const int code = dlt < 0.0 ? (dd > T ? 0 : 1) : (dd >= T ? 3 : 2);
            n_b[0] += code == 0, n_b[1] += code == 1, n_b[2] += code == 2, n_b[3] += code == 3;
            stack_push<0>(st, m, code == 0 ? x : 0.0, code == 1 ? x : 0.0, code == 2 ? x : 0.0, code == 3 ? x : 0.0);
            word |= (unsigned)code << (2 * (m & 15));
            if ((k & 15) == 0) {
                if ((m & 15) == 15) {
                    if (live) reinterpret_cast<unsigned *>(codes_out)[m >> 4] = word;
                    if (codes_out2) reinterpret_cast<unsigned *>(codes_out2)[m >> 4] = word;
                    word = 0;
                }
            } else if ((m & 3) == 3) {
                if (live) codes_out[m >> 2] = (unsigned char)(word >> (2 * (m & 12)));
                if (codes_out2) codes_out2[m >> 2] = (unsigned char)(word >> (2 * (m & 12)));
                if ((m & 15) == 15) word = 0;
            }
        }
    }
    // pad with +0.0 up to the next power of two; the root is then at level log2(P)
    int P = 1, top = 0;
    while (P < k) P <<= 1, ++top;
    for (int m = k; m < P; ++m) stack_push<0>(st, m, 0.0, 0.0, 0.0, 0.0);
    if (live) {
        double r0 = st.a[0], r1 = st.b[0], r2 = st.c[0], r3 = st.d[0];
#pragma unroll
        for (int l = 1; l < LV; ++l)
            if (top == l) r0 = st.a[l], r1 = st.b[l], r2 = st.c[l], r3 = st.d[l];
        A.leafC[0 * A.n_chunks + c] = r0;
        A.leafC[1 * A.n_chunks + c] = r1;
        A.leafC[2 * A.n_chunks + c] = r2;
        A.leafC[3 * A.n_chunks + c] = r3;
#pragma unroll
        for (int b = 0; b < 4; ++b) A.cnt[b * A.n_chunks + c] = n_b[b];
    }
}

// ------------------------------------------------------------------ kernel C at high densities
// Above k = 128 a lane per chunk has too long a walk (and too deep a stack), and on a short list
// it leaves most of the chip idle.  Here one WAVE owns
// a chunk: lane l takes the E = pow2ceil(k)/64 consecutive entries E*l .., folds them through
// the same binary-counter stacks (log2(E) levels, resolved at compile time), and the upper
// levels of the adjacent-pair tree are a butterfly over the lanes (a + b = b + a bit for bit,
// so it does not matter which of a pair of lanes is the left one).  Entries from k on are the
// +0.0 padding of the tree.  Same codes, counts and per-bin roots as k_codes.
template <int E>
__global__ void __launch_bounds__(256) k_codes_wave(CodeArgs A)
{
    constexpr int LV = (E == 1 ? 0 : E == 2 ? 1 : E == 4 ? 2 : E == 8 ? 3 : E == 16 ? 4 : E == 32 ? 5 : 6) + 1;
    const int lane = threadIdx.x & 63, k = A.k;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= A.n_chunks) return;
    const SlChunkDesc d = A.desc[c];
    const double mu = A.tstat[d.tensor].mu;
    const double T = 9.0 * A.tstat[d.tensor].var;      // squared distance of the outer edges (3 sigma)
    unsigned char *const record_codes = A.payload + d.rec_off + 3 * k / 2;
    const float *vin = A.vals + c * k;
    const int m0 = E * lane;

    BinStacksT<LV> st;
#pragma unroll
    for (int l = 0; l < LV; ++l) st.a[l] = st.b[l] = st.c[l] = st.d[l] = 0.0;
    unsigned long long counts = 0;           // four 16-bit counters, bin b in bits 16b..
    unsigned words[E / 16 > 0 ? E / 16 : 1];
#pragma unroll
    for (int w = 0; w < (E / 16 > 0 ? E / 16 : 1); ++w) words[w] = 0u;
    auto entry = [&](int j, float xf) {      // entry j of this lane (j a compile-time constant after unrolling)
        const bool valid = m0 + j < k;
        const double x = (double)xf;
        const double dlt = x - mu;
        const double dd = dlt * dlt;
        const int code = dlt < 0.0 ? (dd > T ? 0 : 1) : (dd >= T ? 3 : 2);
        counts += valid ? 1ull << (16 * code) : 0ull;
        stack_push<0>(st, j, valid && code == 0 ? x : 0.0, valid && code == 1 ? x : 0.0,
                      valid && code == 2 ? x : 0.0, valid && code == 3 ? x : 0.0);
        words[j / 16] |= (valid ? (unsigned)code : 0u) << (2 * (j & 15));
    };
    if constexpr (E == 1) {
        entry(0, m0 < k ? vin[m0] : 0.f);
    } else if constexpr (E == 2) {
        float2 v2 = make_float2(0.f, 0.f);
        if (m0 < k) v2 = *reinterpret_cast<const float2 *>(vin + m0);              // k is a multiple of 4
        entry(0, v2.x);
        entry(1, v2.y);
    } else {
#pragma unroll
        for (int j4 = 0; j4 < E; j4 += 4) {
            float4 v4 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (m0 + j4 < k) v4 = *reinterpret_cast<const float4 *>(vin + m0 + j4);
            entry(j4 + 0, v4.x);
            entry(j4 + 1, v4.y);
            entry(j4 + 2, v4.z);
            entry(j4 + 3, v4.w);
        }
    }
    // the lane's subtree roots, then the levels above them across the lanes: log2(pow2ceil(k) / E)
    // of them (six, except at E = 1, where the padded sequence may be shorter than the wave)
    int levels = 6;
    if constexpr (E == 1) {
        levels = 0;
        while ((1 << levels) < k) ++levels;
    }
    double r0 = st.a[LV - 1], r1 = st.b[LV - 1], r2 = st.c[LV - 1], r3 = st.d[LV - 1];
    r0 = sl_wave_tree(r0, levels), r1 = sl_wave_tree(r1, levels), r2 = sl_wave_tree(r2, levels),
    r3 = sl_wave_tree(r3, levels);
#pragma unroll
    for (int l = 0; l < 6; ++l) counts += sl_partner(counts, l);

    // codes: E/4 bytes per lane at byte E/4 * lane of the code stream (whole bytes: k % 4 == 0)
    const int nbytes = min(E / 4, max(0, (k - m0) / 4));
    auto store_codes = [&](unsigned char *codes_out) __attribute__((always_inline)) {
    if constexpr (E < 4) {
        // 4 / E lanes share a byte, 16 / E lanes a word: OR the lanes' bits together inside the row
        constexpr int LW = 16 / E;                           // lanes per word
        unsigned w = words[0] << (2 * E * (lane & (LW - 1)));
        w |= (unsigned)sl_dpp<SL_DPP_XOR1>((int)w);
        w |= (unsigned)sl_dpp<SL_DPP_XOR2>((int)w);
        w |= (unsigned)sl_dpp<SL_DPP_HALF_MIRROR>((int)w);
        if constexpr (E == 1) w |= (unsigned)sl_dpp<SL_DPP_MIRROR>((int)w);
        if ((k & 15) == 0) {
            if ((lane & (LW - 1)) == 0 && m0 < k) reinterpret_cast<unsigned *>(codes_out)[lane / LW] = w;
        } else {
            constexpr int LB = 4 / E;                        // lanes per byte
            if ((lane & (LB - 1)) == 0 && m0 < k)
                codes_out[lane / LB] = (unsigned char)(w >> (8 * ((lane & (LW - 1)) / LB)));
        }
    } else if ((k & 15) == 0 && nbytes == E / 4) {   // records of whole words: aligned stores
        if constexpr (E == 4) {
            codes_out[lane] = (unsigned char)words[0];
        } else if constexpr (E == 8) {
            reinterpret_cast<unsigned short *>(codes_out)[lane] = (unsigned short)words[0];
        } else {
#pragma unroll
            for (int w = 0; w < E / 16; ++w) reinterpret_cast<unsigned *>(codes_out)[(E / 16) * lane + w] = words[w];
        }
    } else {
#pragma unroll
        for (int b = 0; b < E / 4; ++b)
            if (b < nbytes) codes_out[(E / 4) * lane + b] = (unsigned char)(words[b / 4] >> (8 * (b & 3)));
    }
    };
    store_codes(record_codes);
    if (unsigned char *second = coded_values(A, d)) store_codes(second);
    if (lane == 0) {
        A.leafC[0 * A.n_chunks + c] = r0;
        A.leafC[1 * A.n_chunks + c] = r1;
        A.leafC[2 * A.n_chunks + c] = r2;
        A.leafC[3 * A.n_chunks + c] = r3;
#pragma unroll
        for (int b = 0; b < 4; ++b) A.cnt[b * A.n_chunks + c] = (unsigned)(counts >> (16 * b)) & 0xFFFFu;
    }
}

// ------------------------------------------------------------------ kernel C, other widths
// The same quantizer with 2^BITS uniform bins over [-6 sigma, 6 sigma] (the
// paper's quantization ablation: 1, 3 and 4 bits).  Bin q is
// [c_q, c_(q+1)) sigma around the mean with c_j = 12 j / 2^BITS - 6, the end
// bins open-ended; the code is the number of inner edges the value has
// reached, each edge decided on squares against (c_j * c_j) * var.  The bins
// are handled four at a time (one pass over the chunk's values per group of
// four), so that the per-bin tree stacks stay in registers.
// Is the value at distance dlt from the mean at or beyond inner edge j (1 <= j < 2^BITS)?  The edge
// sits at c_j sigma, c_j = 12 j / 2^BITS - 6 (exact in fp64); decided on squares against (c_j c_j) var.
template <int BITS>
SL_DEV bool edge_reached(int j, double dlt, double dd, double var)
{
    const double cj = (double)j * (12.0 / (double)(1 << BITS)) - 6.0;    // exact: small integer times a power-of-two multiple of 3
    const double Tj = (cj * cj) * var;
    const bool nonneg = dlt >= 0.0;
    return cj < 0.0 ? (nonneg || dd <= Tj) : cj == 0.0 ? nonneg : (nonneg && dd >= Tj);
}

// The code of a value = the number of inner edges it has reached.  The edges ascend, so "reached"
// holds for a prefix of them and the count is found by bisection (BITS decisions instead of 2^BITS - 1).
template <int BITS>
SL_DEV int code_of(double dlt, double var)
{
    const double dd = dlt * dlt;
    int code = 0;
#pragma unroll
    for (int s = BITS - 1; s >= 0; --s) {
        const int mid = code + (1 << s);
        code = edge_reached<BITS>(mid, dlt, dd, var) ? mid : code;
    }
    return code;
}

// One lane per chunk as in k_codes.  The codes are found in the first pass and parked in LDS (a
// word per eight entries); every pass sums NBP bins.
template <int BITS, int LV, int NBP, int WAVES_PER_EU>
__global__ void __launch_bounds__(64 * CODE_WAVES, WAVES_PER_EU) k_codes_b(CodeArgs A)
{
    constexpr int NB = 1 << BITS;
    constexpr int PASSES = (NB + NBP - 1) / NBP;
    constexpr int TC = 32, PITCH = TC + 1;
    extern __shared__ __align__(16) unsigned char codes_lds[];
    const int lane = threadIdx.x & 63, k = A.k;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c0 = ((long long)blockIdx.x * CODE_WAVES + wave) * 64;
    if (c0 >= A.n_chunks) return;
    // per wave: the value tile, then the parked codes (k / 8 words per lane, word w of lane l at [w * 64 + l])
    const bool park = PASSES > 1 && A.park;
    const size_t per_wave = sizeof(float) * 64 * PITCH + (park ? sizeof(unsigned) * 64 * (size_t)(k >> 3) : 0);
    float *tile = reinterpret_cast<float *>(codes_lds + (size_t)wave * per_wave);
    unsigned *parked = reinterpret_cast<unsigned *>(tile + 64 * PITCH);
    const long long c = c0 + lane;
    const bool live = c < A.n_chunks;

    double mu = 0.0, var = 0.0;
    unsigned char *codes_out = nullptr, *codes_out2 = nullptr;
    if (live) {
        const SlChunkDesc d = A.desc[c];
        mu = A.tstat[d.tensor].mu;
        var = A.tstat[d.tensor].var;
        codes_out = A.payload + d.rec_off + 3 * k / 2;
        codes_out2 = coded_values(A, d);
    }
    int P = 1, top = 0;
    while (P < k) P <<= 1, ++top;
    constexpr int LPR = TC / 4;              // lanes that load one row of the tile
    const int lr = lane / LPR, lc = (lane % LPR) * 4;

    for (int pass = 0; pass < PASSES; ++pass) {
        const int q0 = NBP * pass;
        // (four bins to a set of stacks, as in k_codes; NBP = 8: two sets)
        BinStacksT<LV> st, st2;
#pragma unroll
        for (int l = 0; l < LV; ++l) {
            st.a[l] = st.b[l] = st.c[l] = st.d[l] = 0.0;
            st2.a[l] = st2.b[l] = st2.c[l] = st2.d[l] = 0.0;
        }
        unsigned n_b[NBP];
#pragma unroll
        for (int q = 0; q < NBP; ++q) n_b[q] = 0u;
        unsigned bitbuf = 0;                    // codes of 8 entries = BITS bytes
        for (int s0 = 0; s0 < k; s0 += TC) {
            const int ncol = min(TC, k - s0);   // a multiple of 8
            sl_wave_sync();
#pragma unroll
            for (int i = 0; i < LPR; ++i) {
                const int row = (64 / LPR) * i + lr;
                if (c0 + row < A.n_chunks && lc < ncol) {
                    const float4 v = *reinterpret_cast<const float4 *>(A.vals + (c0 + row) * k + s0 + lc);
                    float *t = tile + row * PITCH + lc;
                    t[0] = v.x, t[1] = v.y, t[2] = v.z, t[3] = v.w;
                }
            }
            sl_wave_sync();
            for (int col = 0; col < ncol; ++col) {
                const int m = s0 + col;
                const double x = (double)tile[lane * PITCH + col];
                int code;
                if (pass == 0 || !park) {
                    code = code_of<BITS>(x - mu, var);
                }
                if (pass == 0) {
                    bitbuf |= (unsigned)code << (BITS * (m & 7));
                    if ((m & 7) == 7) {         // k is a multiple of 8
                        if (live) {
#pragma unroll
                            for (int q = 0; q < BITS; ++q)
                                codes_out[(m >> 3) * BITS + q] = (unsigned char)(bitbuf >> (8 * q));
                        }
                        if (codes_out2) {
#pragma unroll
                            for (int q = 0; q < BITS; ++q)
                                codes_out2[(m >> 3) * BITS + q] = (unsigned char)(bitbuf >> (8 * q));
                        }
                        if (park) parked[(m >> 3) * 64 + lane] = bitbuf;
                        bitbuf = 0;
                    }
                } else if (park) {
                    if ((m & 7) == 0) bitbuf = parked[(m >> 3) * 64 + lane];
                    code = (int)((bitbuf >> (BITS * (m & 7))) & (unsigned)(NB - 1));
                }
                const int rel = code - q0;
#pragma unroll
                for (int q = 0; q < NBP; ++q) n_b[q] += rel == q;
                stack_push<0>(st, m, rel == 0 ? x : 0.0, rel == 1 ? x : 0.0, rel == 2 ? x : 0.0, rel == 3 ? x : 0.0);
                if constexpr (NBP > 4)
                    stack_push<0>(st2, m, rel == 4 ? x : 0.0, rel == 5 ? x : 0.0, rel == 6 ? x : 0.0, rel == 7 ? x : 0.0);
            }
        }
        for (int m = k; m < P; ++m) {
            stack_push<0>(st, m, 0.0, 0.0, 0.0, 0.0);
            if constexpr (NBP > 4) stack_push<0>(st2, m, 0.0, 0.0, 0.0, 0.0);
        }
        if (live) {
            double r[8] = {st.a[0], st.b[0], st.c[0], st.d[0], st2.a[0], st2.b[0], st2.c[0], st2.d[0]};
#pragma unroll
            for (int l = 1; l < LV; ++l)
                if (top == l) {
                    r[0] = st.a[l], r[1] = st.b[l], r[2] = st.c[l], r[3] = st.d[l];
                    r[4] = st2.a[l], r[5] = st2.b[l], r[6] = st2.c[l], r[7] = st2.d[l];
                }
#pragma unroll
            for (int q = 0; q < NBP; ++q)
                if (q0 + q < NB) {
                    A.leafC[(long long)(q0 + q) * A.n_chunks + c] = r[q];
                    A.cnt[(long long)(q0 + q) * A.n_chunks + c] = n_b[q];
                }
        }
    }
}

// ------------------------------------------------------------------ kernel D
// One workgroup per (tensor, bin): fixed-tree sum of the bin's leaves, integer
// count, centroid -> LUT[b] in the tensor block's header.
__global__ void __launch_bounds__(RED_THREADS)
k_tensor_lut(const SlTensorDev *tensors, const double *leafC, const unsigned *cnt,
             long long n_chunks_total, int hdr_bytes, int rec_bytes, int nbins, unsigned char *payload,
             unsigned char *coded, int cfix)
{
    __shared__ RedShared sh;
    const SlTensorDev td = tensors[blockIdx.x];
    const int b = blockIdx.y;
    const int tid = threadIdx.x;
    if (tid == 0) sh.cnt[0] = 0ull;
    __syncthreads();
    unsigned long long part = 0;
    for (long long i = tid; i < td.n_chunks; i += RED_THREADS)
        part += cnt[b * n_chunks_total + td.chunk0 + i];
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) part += __shfl_xor(part, s);
    if ((tid & 63) == 0 && part) atomicAdd(&sh.cnt[0], part);   // integer: order-free
    __syncthreads();
    const double Sb = block_tree_sum(leafC + b * n_chunks_total + td.chunk0, td.n_chunks, sh);
    if (tid == 0) {
        const unsigned long long nb = sh.cnt[0];
        float cen = nb ? (float)(Sb / (double)nb) : 0.0f;
        if (cen == 0.0f) cen = 0.0f;        // never -0.0f on the wire
        reinterpret_cast<float *>(payload + td.pay_off)[b] = cen;
        if (coded) reinterpret_cast<float *>(coded + td.cblk_off)[b] = cen;
    }
    // zero the padding that rounds the header (two floats at 1 bit) and the tensor block up to 16 bytes
    if (b == 0 && tid >= nbins && 4 * tid < hdr_bytes) {
        reinterpret_cast<float *>(payload + td.pay_off)[tid] = 0.0f;
        if (coded) reinterpret_cast<float *>(coded + td.cblk_off)[tid] = 0.0f;
    }
    const long long used = hdr_bytes + td.n_chunks * (long long)rec_bytes;
    if (b == 0 && tid < td.block_bytes - used) payload[td.pay_off + used + tid] = 0;
    // the same table and padding in the coded buffer's block
    const long long cused = (td.cfix_off - td.cblk_off) + td.n_chunks * (long long)cfix;
    if (coded && b == 0 && tid < td.cblk_bytes - cused) coded[td.cblk_off + cused + tid] = 0;
}

// Unquantized values: there is no table, only the block padding is left to write.
__global__ void __launch_bounds__(64)
k_pad_blocks(const SlTensorDev *tensors, int rec_bytes, unsigned char *payload, unsigned char *coded, int cfix)
{
    const SlTensorDev td = tensors[blockIdx.x];
    const long long used = td.n_chunks * (long long)rec_bytes;
    if ((long long)threadIdx.x < td.block_bytes - used) payload[td.pay_off + used + threadIdx.x] = 0;
    const long long cused = (td.cfix_off - td.cblk_off) + td.n_chunks * (long long)cfix;
    if (coded && (long long)threadIdx.x < td.cblk_bytes - cused) coded[td.cblk_off + cused + threadIdx.x] = 0;
}

// ------------------------------------------------------------------ kernel E
struct ResidualArgs {
    const SlChunkDesc *desc;
    const float *vals;              // the selected values a, or null: read them from e
    const unsigned char *payload;
    float *e;
    long long n_chunks;
    int k, bits, hdr_bytes, rec_bytes;
};

__global__ void __launch_bounds__(256) k_residual(ResidualArgs A)
{
    const int lane = threadIdx.x & 63, k = A.k;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= A.n_chunks) return;
    const SlChunkDesc d = A.desc[c];
    const float *lut = reinterpret_cast<const float *>(A.payload + sl_lut_off(d, A.hdr_bytes, A.rec_bytes));
    const unsigned char *rec = A.payload + d.rec_off;
    const unsigned char *codes = rec + 3 * k / 2;       // or the k fp32 values (4-byte aligned)
    float *ec = A.e + d.base;
    for (int m = lane; m < k; m += 64) {
        const int b = (3 * m) >> 1;
        const unsigned w = (unsigned)rec[b] | ((unsigned)rec[b + 1] << 8);
        const unsigned j = (m & 1) ? (w >> 4) : (w & 0xFFFu);
        const float q = A.bits == 32 ? reinterpret_cast<const float *>(codes)[m]
                                     : lut[sl_code_at(codes, m, A.bits)];
        float *dst = ec + ((j >> 6) * (unsigned)d.stride + (j & 63u));
        const float a = A.vals ? A.vals[c * k + m] : *dst;
        *dst = a - q;
    }
}

}  // namespace

static int check_launch()
{
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    return SL_OK;
}

static int launch_residual(const sl_plan *p, float *e, const float *vals, const unsigned char *payload,
                           hipStream_t st)
{
    ResidualArgs R;
    R.desc = p->d_desc;
    R.vals = vals;
    R.payload = payload;
    R.e = e;
    R.k = p->k;
    R.bits = p->bits;
    R.hdr_bytes = p->hdr_bytes;
    R.rec_bytes = p->rec_bytes;
    R.n_chunks = p->n_chunks;
    const int wpb = 4;
    const unsigned nblk = (unsigned)((p->n_chunks + wpb - 1) / wpb);
    hipLaunchKernelGGL(k_residual, dim3(nblk), dim3(64 * wpb), 0, st, R);
    return check_launch();
}

int slk_residual(const sl_plan *p, float *e, const unsigned char *payload, hipStream_t st)
{
    if (p->n_chunks == 0) return SL_OK;
    return launch_residual(p, e, nullptr, payload, st);
}

int slk_quantize(const sl_plan *p, float *e, int skip_residual, unsigned char *payload, unsigned char *coded,
                 unsigned char *ws, hipStream_t st)
{
    if (p->n_chunks == 0) return SL_OK;
    const int k = p->k;
    const float *vals = reinterpret_cast<const float *>(ws + p->ws_vals);
    double *leafA = reinterpret_cast<double *>(ws + p->ws_leafA);
    double *leafC = reinterpret_cast<double *>(ws + p->ws_leafC);
    unsigned *cnt = reinterpret_cast<unsigned *>(ws + p->ws_cnt);
    SlTensorStat *tstat = reinterpret_cast<SlTensorStat *>(ws + p->ws_tstat);
    int rc;

    if (p->bits == 32) {
        // nothing to quantize: kernel A wrote the values into the records
        hipLaunchKernelGGL(k_pad_blocks, dim3(p->n_tensors), dim3(64), 0, st, p->d_tensors, p->rec_bytes,
                           payload, coded, p->cg.cfix);
        if ((rc = check_launch())) return rc;
        sl_prof_mark(p, SL_PROF_LUT, st);
        if (!skip_residual) {
            if ((rc = launch_residual(p, e, vals, payload, st))) return rc;
            sl_prof_mark(p, SL_PROF_RESIDUAL, st);
        }
        return SL_OK;
    }

    hipLaunchKernelGGL(k_tensor_stats, dim3(p->n_tensors), dim3(RED_THREADS), 0, st, p->d_tensors,
                       leafA, (long long)p->n_chunks, k, tstat);
    if ((rc = check_launch())) return rc;
    sl_prof_mark(p, SL_PROF_STATS, st);

    CodeArgs C;
    C.desc = p->d_desc;
    C.tstat = tstat;
    C.vals = vals;
    C.leafC = leafC;
    C.cnt = cnt;
    C.payload = payload;
    C.n_chunks = p->n_chunks;
    C.k = k;
    C.coded = coded;
    C.tensors = p->d_tensors;
    C.cfix = p->cg.cfix;
    C.rem_bytes = p->cg.rem_bytes;
    C.park = 0;
    const long long per_block = 64ll * CODE_WAVES;
    const unsigned nblk = (unsigned)((p->n_chunks + per_block - 1) / per_block);
    // (the list length is a field of the plan, sl_plan_set_codes_wave_below: both kernels write the same bytes)
    const bool by_wave = k >= SL_CODES_WAVE_FROM || p->n_chunks < p->codes_wave_below;
    switch (p->bits) {
        case 1:
        case 3:
        case 4: {
            // stack depth by k as in k_codes; bins per pass: as many as the registers hold next to it
            const int depth = k <= 64 ? 7 : k <= 256 ? 9 : 13;
            const int nbp = p->bits == 1 ? 2 : 4;     // (eight at a time is no faster: the pushes per bin are the cost)
            const int passes = ((1 << p->bits) + nbp - 1) / nbp;
            C.park = passes > 1 && k <= 512;          // 32 KB of LDS per workgroup at most
            const size_t lds = CODE_WAVES * (sizeof(float) * 64 * 33 + (C.park ? sizeof(unsigned) * 64 * (size_t)(k >> 3) : 0));
            const dim3 g(nblk), b(64 * CODE_WAVES);
#define SL_CODES_B(BITS, LV, NBP, WPE) hipLaunchKernelGGL((k_codes_b<BITS, LV, NBP, WPE>), g, b, lds, st, C)
            if (p->bits == 1) {
                if (depth == 7) SL_CODES_B(1, 7, 2, 4);
                else if (depth == 9) SL_CODES_B(1, 9, 2, 4);
                else SL_CODES_B(1, 13, 2, 2);
            } else if (p->bits == 3) {
                if (depth == 7) SL_CODES_B(3, 7, 4, 4);
                else if (depth == 9) SL_CODES_B(3, 9, 4, 3);
                else SL_CODES_B(3, 13, 4, 2);
            } else {
                if (depth == 7) SL_CODES_B(4, 7, 4, 4);
                else if (depth == 9) SL_CODES_B(4, 9, 4, 3);
                else SL_CODES_B(4, 13, 4, 2);
            }
#undef SL_CODES_B
            break;
        }
        default:
            if (k <= 64 && !by_wave) {
                hipLaunchKernelGGL((k_codes<7, 32, 4>), dim3(nblk), dim3(64 * CODE_WAVES), 0, st, C);
            } else if (k <= 256 && !by_wave) {
                hipLaunchKernelGGL((k_codes<9, 32, 4>), dim3(nblk), dim3(64 * CODE_WAVES), 0, st, C);
            } else if (!by_wave) {
                hipLaunchKernelGGL((k_codes<13, 64, 2>), dim3(nblk), dim3(64 * CODE_WAVES), 0, st, C);
            } else {
                // a wave per chunk, E = pow2ceil(k) / 64 entries per lane
                const dim3 wgrid((unsigned)((p->n_chunks + 3) / 4)), wblock(256);
                if (k <= 64) hipLaunchKernelGGL(k_codes_wave<1>, wgrid, wblock, 0, st, C);
                else if (k <= 128) hipLaunchKernelGGL(k_codes_wave<2>, wgrid, wblock, 0, st, C);
                else if (k <= 256) hipLaunchKernelGGL(k_codes_wave<4>, wgrid, wblock, 0, st, C);
                else if (k <= 512) hipLaunchKernelGGL(k_codes_wave<8>, wgrid, wblock, 0, st, C);
                else if (k <= 1024) hipLaunchKernelGGL(k_codes_wave<16>, wgrid, wblock, 0, st, C);
                else if (k <= 2048) hipLaunchKernelGGL(k_codes_wave<32>, wgrid, wblock, 0, st, C);
                else hipLaunchKernelGGL(k_codes_wave<64>, wgrid, wblock, 0, st, C);
            }
            break;
    }
    if ((rc = check_launch())) return rc;
    sl_prof_mark(p, SL_PROF_CODES, st);

    hipLaunchKernelGGL(k_tensor_lut, dim3(p->n_tensors, 1 << p->bits), dim3(RED_THREADS), 0, st,
                       p->d_tensors, leafC, cnt, (long long)p->n_chunks, p->hdr_bytes, p->rec_bytes,
                       1 << p->bits, payload, coded, p->cg.cfix);
    if ((rc = check_launch())) return rc;
    sl_prof_mark(p, SL_PROF_LUT, st);

    if (!skip_residual) {
        if ((rc = launch_residual(p, e, vals, payload, st))) return rc;
        sl_prof_mark(p, SL_PROF_RESIDUAL, st);
    }
    return SL_OK;
}
