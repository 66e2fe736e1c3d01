// sl_decompress_avg_apply: dequantise R workers' sparse payloads, average and
// take the outer SGD step in one pass over theta (Algorithm 1, "Aggregate +
// Outer Update"; Eq. (2) lines 3-4), and the stand-alone record encoder
// sl_pack_indices (12-bit index fields + 2-bit codes).
//
// One wavefront owns one chunk.  The dense average never exists in HBM: the
// chunk's fp32 accumulators live in LDS (16 KB, or one half of the chunk at a
// time), the R records (7k/4 bytes each) are staged into LDS with coalesced
// loads, entries of one worker are distinct positions so they are added without
// conflicts, workers are added in the order r = 0..R-1, and theta streams
// through registers once (8 bytes per element of HBM traffic plus R*7k/4 bytes
// per chunk).
#include "sl_device.h"
#include "sl_internal.h"

namespace {

// When there is much to decode per chunk (R*k entries) at small k, the chunk is
// aggregated in NH = 2 halves of 32 rows (local indices below / from 2048): 8 KB of
// accumulators per wave instead of 16, so that more waves - and more bytes of
// theta in flight - fit a compute unit while the decode runs.  With little to
// decode, and from k = 256 (cheaper decode, records staged 4 KB at a time), one
// pass (NH = 1) is faster.
#ifndef SL_APPLY_HALVES_FROM
#define SL_APPLY_HALVES_FROM 1536   // R*k from which two halves pay (measured)
#endif

#ifndef SL_APPLY_OCTETS_FROM
#define SL_APPLY_OCTETS_FROM 256   // k from which a lane decodes eight entries at a time
#endif
#ifndef SL_APPLY_QUADS_FROM
#define SL_APPLY_QUADS_FROM 136    // ... or four (2-bit records with many entries to decode per chunk)
#endif
#ifndef SL_APPLY_QUADS_ENTRIES
#define SL_APPLY_QUADS_ENTRIES 2048     // ... R * k from which that holds below k = 256
#endif
#ifndef SL_APPLY_PF1
#define SL_APPLY_PF1 16     // words per lane fetched ahead of the theta loads on the entry-by-entry route (2-bit codes)
#endif
#ifndef SL_APPLY_STAGE_U
#define SL_APPLY_STAGE_U 8    // words per lane loaded together while records are staged
#endif
#ifndef SL_APPLY_BIG_STAGE
#define SL_APPLY_BIG_STAGE 4096   // staging bytes on the eight-entry route, and when one record is larger than 1 KB
#endif

// pointers into global memory, for addresses that are put together from integers
typedef const unsigned char __attribute__((address_space(1))) *sl_gbytes;
typedef const unsigned __attribute__((address_space(1))) *sl_gwords;

// acc[j] += q in LDS, as a read, an fp32 add and a write.  (The LDS unit's own fp32 add gives the
// same bits, subnormal sums included, but at a fraction of the rate: 2.35 -> 2.45 ms at k = 64 and
// several times slower from k = 256.)
SL_DEV void acc_add(float *acc, unsigned j, float q) { acc[j] = acc[j] + q; }

struct ApplyArgs {
    const SlChunkDesc *desc;
    float *theta;
    float *mom;              // global outer momentum buffer (Nesterov variant), else null
    float mu;
    float neg_lr, inv_R;
    int R, k;
    int bits, hdr_bytes, rec_bytes;   // value width and the sizes that follow from it
    int batch;               // records staged per round
    int quads;               // eight-entry route, 2-bit format: four entries per lane instead (up to k = 256: a
                             // worker's record then spans up to 64 lanes instead of 32, in one round)
    // x / d for the staging loops without a division: __umulhi(x, floor(2^32 / d) + 1) is
    // exact while x * d < 2^32 (x < 16384 here); d = words per (table + record padded to whole words)
    unsigned magic_src;
    int lds_per_wave;
    long long n_chunks;
    const unsigned char *payload[SL_MAX_WORKERS];
};

// One wave per chunk, several independent waves (adjacent chunks) per workgroup.
// TWO_BIT: the 2-bit format, its sizes compile-time constants; otherwise any
// width (table of 2^bits entries, or fp32 values).
// NESTEROV: DiLoCo's global outer momentum on top of the aggregate (Eq. (1);
// appendix algorithm "Outer step for DiLoCo+Top-k[+EF]"): m <- mu*m + avg,
// d <- avg + mu*m, theta <- theta - lr*d at every element of the chunk.
// ROUTE: how a staged record's entries reach the accumulators.
//   0 (k <= 128, one pass): the entries of several workers are decoded ahead of the additions;
//   1: entry by entry, one worker at a time;
//   2 (k >= 256, a multiple of 8): a lane decodes eight consecutive entries from whole words.
// The routes are separate instantiations, so that none pays for another's registers.
template <bool TWO_BIT, bool NESTEROV, int NH, int ROUTE>
__global__ void __launch_bounds__(256) k_apply(ApplyArgs A)
{
    constexpr bool SMALLK = ROUTE == 0, OCTETS = ROUTE == 2;
    static_assert(ROUTE == 1 || NH == 1, "two halves go entry by entry");
    constexpr int ACC_FLOATS = SL_CHUNK / NH, ROWS4 = 16 / NH;   // accumulators, 16-byte accesses per lane
    extern __shared__ __align__(16) unsigned char smem_all[];
    const int lane = threadIdx.x & 63, k = A.k;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= A.n_chunks) return;
    unsigned char *smem = smem_all + (size_t)wave * A.lds_per_wave;
    float *acc = reinterpret_cast<float *>(smem);                    // the chunk, or one half of it
    unsigned char *stage = smem + ACC_FLOATS * sizeof(float);
    const SlChunkDesc d = A.desc[c];
    const int bits = TWO_BIT ? 2 : A.bits;
    const int hdr = TWO_BIT ? 16 : A.hdr_bytes, hdr_words = hdr >> 2;
    const int rec_bytes = TWO_BIT ? 7 * k / 4 : A.rec_bytes;
    const int rec_pad = ((rec_bytes + 3) & ~3) + hdr;                // staging pitch: LUT + record
    const long long rec_off = d.rec_off, lut_off = sl_lut_off(d, hdr, rec_bytes);

    float *tc = A.theta + d.base;
    const int lr = lane >> 4, lc = (lane & 15) * 4;
    const unsigned stride = (unsigned)d.stride;
    const bool full = d.flags & SLC_FULL;

    // Word w of a batch's staging area: worker r = w / wpr, word q of (LUT, record padded to words)
    const int wpr = rec_pad >> 2;
    // Worker r's payload pointer where r differs from lane to lane: lane l keeps worker l's
    // pointer (there are at most as many workers as lanes) and the others read it across
    // lanes.  Indexing the kernel argument with a per-lane r instead costs a dependent vector
    // load of the pointer in front of every access.  Called by all 64 lanes together.
    static_assert(SL_MAX_WORKERS <= 64, "one payload pointer per lane");
    const unsigned long long my_ptr = reinterpret_cast<unsigned long long>(A.payload[lane]);
    // (the pointer comes back as an integer: it is cast to the global address space by hand, a
    // generic pointer would turn every access into a flat load that LDS waits have to sit out)
    auto payload_of = [&](int r) -> sl_gbytes {
        const unsigned lo = (unsigned)__builtin_amdgcn_ds_bpermute(4 * r, (int)(unsigned)my_ptr);
        const unsigned hi = (unsigned)__builtin_amdgcn_ds_bpermute(4 * r, (int)(unsigned)(my_ptr >> 32));
        return reinterpret_cast<sl_gbytes>(((unsigned long long)hi << 32) | lo);
    };
    // Word w of workers r_first.. taken as one run of (LUT, record) blocks, or 0 beyond `nw`.  A
    // record that is not a whole number of words lies at any byte of the payload: its word i is
    // put together from the two aligned words that hold its bytes (only words that hold bytes
    // of the record are read).
    const unsigned sh = (unsigned)(rec_off & 3);
    const long long a0 = rec_off & ~3ll, a1 = (rec_off + rec_bytes + 3) & ~3ll;
    auto src_word = [&](int r_first, int w, int nw) -> unsigned {
        const bool valid = w < nw;
        const int r = valid ? (int)__umulhi((unsigned)w, A.magic_src) : 0, q = w - r * wpr;
        const sl_gbytes p = payload_of(r_first + r);
        unsigned v = 0;
        if (valid) {
            if (q < hdr_words) {
                v = reinterpret_cast<sl_gwords>(p + lut_off)[q];
            } else {
                const int i = q - hdr_words;
                const sl_gwords src = reinterpret_cast<sl_gwords>(p + a0) + i;
                v = src[0];
                if (sh != 0u) v = __builtin_amdgcn_alignbyte(a0 + 4ll * i + 4 < a1 ? src[1] : 0u, v, sh);
            }
        }
        return v;
    };
    // The first 64*PF words of the first batch (all of it for R*(16 + 7k/4) <= 2 KB:
    // R = 8 up to k = 128, R = 16 up to k = 64) are fetched into registers BEFORE the
    // theta loads, so that they arrive with the chunk instead of costing a second round
    // trip to memory behind it.  (As compiled, the wait in front of the words' parking
    // below is for every outstanding load, theta included: the parking sits in a loop.
    // With that wait made exact the decode overlaps the theta loads, and nothing is
    // gained - this kernel's decode is short - so the simpler form stays.)
    // (wider records at other widths: 3 KB; many workers at small k, the entry-by-entry route, and
    // the eight-entry route: 4 KB, which is all that is staged at a time there)
    constexpr int PF = ROUTE == 2 ? 16 : !TWO_BIT ? 12 : ROUTE == 1 ? SL_APPLY_PF1 : 8;
    unsigned pf[PF];
    const int nb0 = min(A.batch, A.R);
#pragma unroll
    for (int u = 0; u < PF; ++u) pf[u] = src_word(0, lane + 64 * u, nb0 * wpr);

    sl_f4 th[16], mo[NESTEROV ? 16 : 1];
    float *mc = NESTEROV ? A.mom + d.base : nullptr;
    if (full) {
        const unsigned o0 = 4u * (lr * stride + lc), step = 16u * stride;
#pragma unroll
        for (int i = 0; i < 16; ++i) th[i] = sl_load_stream_at(tc, i * step, o0);
        if constexpr (NESTEROV) {
#pragma unroll
            for (int i = 0; i < 16; ++i) mo[i] = sl_load_stream_at(mc, i * step, o0);
        }
    } else {
        // partial chunk: the same loads up front, 16 bytes where a lane's four columns lie inside
        // the tensor (rows need no alignment), element by element at the edge, nothing outside
        const int rows = d.rows, cols = d.cols, last_cols = d.last_cols;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = 4 * i + lr;
            const int lim = row < rows - 1 ? cols : (row == rows - 1 ? last_cols : 0);
            const unsigned o0 = row * stride + lc;
            th[i] = sl_f4{0.f, 0.f, 0.f, 0.f};
            if constexpr (NESTEROV) mo[i] = sl_f4{0.f, 0.f, 0.f, 0.f};
            if (lc + 3 < lim) {
                th[i] = sl_load_stream_u(tc + o0);
                if constexpr (NESTEROV) mo[i] = sl_load_stream_u(mc + o0);
            } else {
#pragma unroll
                for (int cc = 0; cc < 4; ++cc)
                    if (lc + cc < lim) {
                        th[i][cc] = tc[o0 + cc];
                        if constexpr (NESTEROV) mo[i][cc] = mc[o0 + cc];
                    }
            }
        }
    }

    const bool single = A.R <= A.batch;      // every record fits the staging area at once
#pragma unroll
    for (int h = 0; h < NH; ++h) {
#pragma unroll
        for (int i = 0; i < ROWS4; ++i)
            reinterpret_cast<float4 *>(acc)[i * 64 + lane] = make_float4(0.f, 0.f, 0.f, 0.f);

        for (int r0 = 0; r0 < A.R; r0 += A.batch) {
            const int nb = min(A.batch, A.R - r0);
            sl_wave_sync();
            if (h == 0 || !single) {
                const int nw = nb * wpr;
                int wb = 0;                       // wave-uniform: word wb + lane is this lane's next
                if (r0 == 0 && h == 0) {
#pragma unroll
                    for (int u = 0; u < PF; ++u) {
                        const int w = lane + 64 * u;
                        // (the staging pitch is wpr words: word w lands at w)
                        if (w < nw) reinterpret_cast<unsigned *>(stage)[w] = pf[u];
                    }
                    wb = 64 * PF;
                }
                // the rest: SU words per lane are loaded before the first of them is parked in LDS
                constexpr int SU = SMALLK ? 1 : SL_APPLY_STAGE_U;   // (small k: little or nothing is left)
                for (; wb < nw; wb += 64 * SU) {
                    unsigned v[SU];
#pragma unroll
                    for (int u = 0; u < SU; ++u) v[u] = src_word(r0, wb + 64 * u + lane, nw);
#pragma unroll
                    for (int u = 0; u < SU; ++u) {
                        const int w = wb + 64 * u + lane;
                        if (w < nw) reinterpret_cast<unsigned *>(stage)[w] = v[u];
                    }
                }
                sl_wave_sync();
            }
            // One entry of a staged record: local index (0xFFFF for none) and value.
            auto decode = [&](int r, int m, unsigned &j, float &q) {
                const float *lutp = reinterpret_cast<const float *>(stage + r * rec_pad);
                const unsigned char *rec = stage + r * rec_pad + hdr;
                const unsigned char *codes = rec + 3 * k / 2;   // or the k fp32 values (4-byte aligned)
                const int b = (3 * m) >> 1;
                const unsigned w = (unsigned)rec[b] | ((unsigned)rec[b + 1] << 8);
                j = (m & 1) ? (w >> 4) : (w & 0xFFFu);
                if (TWO_BIT) q = lutp[(codes[m >> 2] >> (2 * (m & 3))) & 3u];
                else if (bits == 32) q = reinterpret_cast<const float *>(codes)[m];
                else q = lutp[sl_code_at(codes, m, bits)];
            };
            if constexpr (SMALLK) {
                // The entries of up to eight workers are decoded first (independent LDS reads,
                // all in flight together), then added worker by worker: the additions form a
                // chain of LDS round trips, the decoding no longer sits inside it.
                for (int rb = 0; rb < nb; rb += 8) {
                    unsigned jj[8][2];
                    float qq[8][2];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
#pragma unroll
                        for (int s2 = 0; s2 < 2; ++s2) {
                            const int m = lane + 64 * s2;
                            jj[u][s2] = 0xFFFFu;
                            qq[u][s2] = 0.0f;
                            if (rb + u < nb && m < k) decode(rb + u, m, jj[u][s2], qq[u][s2]);
                        }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        if (rb + u < nb) {
#pragma unroll
                            for (int s2 = 0; s2 < 2; ++s2) {
                                const unsigned j = jj[u][s2];
                                if (j != 0xFFFFu && (NH == 1 || (int)(j >> 11) == h))
                                    acc_add(acc, j & (ACC_FLOATS - 1), qq[u][s2]);
                            }
                            sl_wave_sync();   // worker r is complete before worker r+1 is added
                        }
                    }
                }
            } else if constexpr (OCTETS) {
                // Eight consecutive entries per lane: their indices are three aligned words
                // of the record and their codes `bits` bytes, so a lane decodes them with 4
                // LDS reads instead of 24 and a fraction of the arithmetic.  The positions
                // of one record are distinct: the eight accumulator reads, then the eight
                // writes, are issued together.
                for (int r = 0; r < nb; ++r) {
                    const unsigned char *base = stage + r * rec_pad;
                    const float *lutp = reinterpret_cast<const float *>(base);
                    const unsigned *iw = reinterpret_cast<const unsigned *>(base + hdr);
                    const unsigned char *codes = base + hdr + 3 * k / 2;
                    float l0 = 0.f, l1 = 0.f, l2 = 0.f, l3 = 0.f;
                    if (TWO_BIT) l0 = lutp[0], l1 = lutp[1], l2 = lutp[2], l3 = lutp[3];
                    if (TWO_BIT && A.quads) {
                        // four consecutive entries = 48 bits that start at bit 0 or 16 of a word
                        for (int q = lane; q < (k >> 2); q += 64) {
                            const int wi = (3 * q) >> 1;
                            const unsigned wa = iw[wi], wb = iw[wi + 1], sh = 16u * (q & 1);
                            const unsigned lo = __builtin_amdgcn_alignbit(wb, wa, sh), hi = wb >> sh;
                            unsigned jq[4];
                            jq[0] = lo & 0xFFFu;
                            jq[1] = (lo >> 12) & 0xFFFu;
                            jq[2] = (lo >> 24) | ((hi & 0xFu) << 8);
                            jq[3] = (hi >> 4) & 0xFFFu;
                            const unsigned cw = codes[q];
                            float qv[4], tq[4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const unsigned cde = cw >> (2 * e);
                                const float lo_v = (cde & 1u) ? l1 : l0, hi_v = (cde & 1u) ? l3 : l2;
                                qv[e] = (cde & 2u) ? hi_v : lo_v;
                            }
#pragma unroll
                            for (int e = 0; e < 4; ++e) tq[e] = acc[jq[e] & (ACC_FLOATS - 1)];
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[jq[e] & (ACC_FLOATS - 1)] = tq[e] + qv[e];
                        }
                        sl_wave_sync();       // worker r is complete before worker r+1 is added
                        continue;
                    }
                    for (int o = lane; o < (k >> 3); o += 64) {
                        const unsigned w0 = iw[3 * o], w1 = iw[3 * o + 1], w2 = iw[3 * o + 2];
                        unsigned jj[8];
                        jj[0] = w0 & 0xFFFu;
                        jj[1] = (w0 >> 12) & 0xFFFu;
                        jj[2] = (w0 >> 24) | ((w1 & 0xFu) << 8);
                        jj[3] = (w1 >> 4) & 0xFFFu;
                        jj[4] = (w1 >> 16) & 0xFFFu;
                        jj[5] = (w1 >> 28) | ((w2 & 0xFFu) << 4);
                        jj[6] = (w2 >> 8) & 0xFFFu;
                        jj[7] = w2 >> 20;
                        float qq[8];
                        if (TWO_BIT) {
                            const unsigned cw = reinterpret_cast<const unsigned short *>(codes)[o];
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                const unsigned cde = cw >> (2 * e);
                                const float lo = (cde & 1u) ? l1 : l0, hi = (cde & 1u) ? l3 : l2;
                                qq[e] = (cde & 2u) ? hi : lo;
                            }
                        } else if (bits == 32) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) qq[e] = reinterpret_cast<const float *>(codes)[8 * o + e];
                        } else {
                            unsigned cw = 0;
                            for (int b = 0; b < bits; ++b) cw |= (unsigned)codes[o * bits + b] << (8 * b);
#pragma unroll
                            for (int e = 0; e < 8; ++e) qq[e] = lutp[(cw >> (e * bits)) & ((1u << bits) - 1u)];
                        }
                        float t[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) t[e] = acc[jj[e] & (ACC_FLOATS - 1)];
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (NH == 1 || (int)(jj[e] >> 11) == h)
                                acc[jj[e] & (ACC_FLOATS - 1)] = t[e] + qq[e];
                    }
                    sl_wave_sync();       // worker r is complete before worker r+1 is added
                }
            } else {
                for (int r = 0; r < nb; ++r) {
                    for (int m = lane; m < k; m += 64) {
                        unsigned j;
                        float q;
                        decode(r, m, j, q);
                        if (NH == 1 || (int)(j >> 11) == h)         // this half's entries
                            acc_add(acc, j & (ACC_FLOATS - 1), q);
                    }
                    sl_wave_sync();           // worker r is complete before worker r+1 is added
                }
            }
        }

        if (full) {
            const unsigned o0 = 4u * (lr * stride + lc), step = 16u * stride;
#pragma unroll
            for (int i8 = 0; i8 < ROWS4; ++i8) {
                const int i = ROWS4 * h + i8;
                const float4 a = reinterpret_cast<const float4 *>(acc)[i8 * 64 + lane];
                sl_f4 g;
                g.x = a.x * A.inv_R, g.y = a.y * A.inv_R, g.z = a.z * A.inv_R, g.w = a.w * A.inv_R;
                if constexpr (NESTEROV) {
                    sl_f4 m = mo[i];
                    m.x = fmaf(A.mu, m.x, g.x), m.y = fmaf(A.mu, m.y, g.y);
                    m.z = fmaf(A.mu, m.z, g.z), m.w = fmaf(A.mu, m.w, g.w);
                    sl_store_stream_at(mc, i * step, o0, m);
                    g.x = fmaf(A.mu, m.x, g.x), g.y = fmaf(A.mu, m.y, g.y);
                    g.z = fmaf(A.mu, m.z, g.z), g.w = fmaf(A.mu, m.w, g.w);
                }
                sl_f4 v = th[i];
                v.x = fmaf(A.neg_lr, g.x, v.x);
                v.y = fmaf(A.neg_lr, g.y, v.y);
                v.z = fmaf(A.neg_lr, g.z, v.z);
                v.w = fmaf(A.neg_lr, g.w, v.w);
                sl_store_stream_at(tc, i * step, o0, v);
            }
        } else {
            const int rows = d.rows, cols = d.cols, last_cols = d.last_cols;
#pragma unroll
            for (int i8 = 0; i8 < ROWS4; ++i8) {
                const int i = ROWS4 * h + i8, row = 4 * i + lr;
                const int lim = row < rows - 1 ? cols : (row == rows - 1 ? last_cols : 0);
                const unsigned o0 = row * stride + lc;
                const float4 a = reinterpret_cast<const float4 *>(acc)[i8 * 64 + lane];
                sl_f4 g;
                g.x = a.x * A.inv_R, g.y = a.y * A.inv_R, g.z = a.z * A.inv_R, g.w = a.w * A.inv_R;
                sl_f4 m = sl_f4{0.f, 0.f, 0.f, 0.f};
                if constexpr (NESTEROV) {
                    m = mo[i];
                    m.x = fmaf(A.mu, m.x, g.x), m.y = fmaf(A.mu, m.y, g.y);
                    m.z = fmaf(A.mu, m.z, g.z), m.w = fmaf(A.mu, m.w, g.w);
                    g.x = fmaf(A.mu, m.x, g.x), g.y = fmaf(A.mu, m.y, g.y);
                    g.z = fmaf(A.mu, m.z, g.z), g.w = fmaf(A.mu, m.w, g.w);
                }
                sl_f4 v = th[i];
                v.x = fmaf(A.neg_lr, g.x, v.x), v.y = fmaf(A.neg_lr, g.y, v.y);
                v.z = fmaf(A.neg_lr, g.z, v.z), v.w = fmaf(A.neg_lr, g.w, v.w);
                if (lc + 3 < lim) {
                    if constexpr (NESTEROV) sl_store_stream_u(mc + o0, m);
                    sl_store_stream_u(tc + o0, v);
                } else {
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc)
                        if (lc + cc < lim) {
                            if constexpr (NESTEROV) mc[o0 + cc] = m[cc];
                            tc[o0 + cc] = v[cc];
                        }
                }
            }
        }
    }
}

// Payload check: every record's indices strictly ascending and inside the
// chunk's valid region.  One wave per chunk; a violation sets *flag.
__global__ void __launch_bounds__(256)
k_validate(const SlChunkDesc *desc, long long n_chunks, int k, const unsigned char *payload, int *flag)
{
    const int lane = threadIdx.x & 63;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= n_chunks) return;
    const SlChunkDesc d = desc[c];
    const unsigned char *rec = payload + d.rec_off;
    bool bad = false;
    for (int m = lane; m < k; m += 64) {
        const int b = (3 * m) >> 1;
        const unsigned w = (unsigned)rec[b] | ((unsigned)rec[b + 1] << 8);
        const int j = (int)((m & 1) ? (w >> 4) : (w & 0xFFFu));
        int prev = -1;
        if (m > 0) {
            const int bp = (3 * (m - 1)) >> 1;
            const unsigned wp = (unsigned)rec[bp] | ((unsigned)rec[bp + 1] << 8);
            prev = (int)(((m - 1) & 1) ? (wp >> 4) : (wp & 0xFFFu));
        }
        const int row = j >> 6, col = j & 63;
        const int lim = row < d.rows - 1 ? d.cols : (row == d.rows - 1 ? d.last_cols : 0);
        bad |= j <= prev || col >= lim;
    }
    if (sl_ballot(bad) && lane == 0) atomicOr(flag, 1);
}

// One thread per output byte of the record stream.
__global__ void __launch_bounds__(256)
k_pack(const uint16_t *idx, const uint8_t *codes, long long n_chunks, int k, unsigned char *out)
{
    const long long rec_bytes = (long long)7 * k / 4;
    const long long total = n_chunks * rec_bytes;
    const int nidx = 3 * k / 2;
    for (long long o = (long long)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (long long)gridDim.x * blockDim.x) {
        const long long c = o / rec_bytes;
        const int b = (int)(o - c * rec_bytes);
        unsigned v;
        if (b < nidx) {
            const int bit0 = 8 * b, m = bit0 / 12, sh = bit0 - 12 * m;   // sh = 0, 4 or 8
            v = ((unsigned)idx[c * k + m] & 0xFFFu) >> sh;
            if (sh == 8 && m + 1 < k) v |= ((unsigned)idx[c * k + m + 1] & 0xFFFu) << 4;
        } else {
            const int m0 = 4 * (b - nidx);
            v = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) v |= ((unsigned)codes[c * k + m0 + q] & 3u) << (2 * q);
        }
        out[o] = (unsigned char)v;
    }
}

// Record encoder for any value width: one thread per output byte; the tail of
// a record is a little-endian stream of `bits`-wide codes, or the fp32 values.
__global__ void __launch_bounds__(256)
k_pack_bits(const uint16_t *idx, const uint8_t *codes, const float *values, long long n_chunks, int k,
            int bits, unsigned char *out)
{
    const long long rec_bytes = sl_rec_bytes(k, bits);
    const long long total = n_chunks * rec_bytes;
    const int nidx = 3 * k / 2;
    for (long long o = (long long)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (long long)gridDim.x * blockDim.x) {
        const long long c = o / rec_bytes;
        const int b = (int)(o - c * rec_bytes);
        unsigned v;
        if (b < nidx) {
            const int bit0 = 8 * b, m = bit0 / 12, sh = bit0 - 12 * m;
            v = ((unsigned)idx[c * k + m] & 0xFFFu) >> sh;
            if (sh == 8 && m + 1 < k) v |= ((unsigned)idx[c * k + m + 1] & 0xFFFu) << 4;
        } else if (bits == 32) {
            const int q = b - nidx;
            v = __float_as_uint(values[c * k + (q >> 2)]) >> (8 * (q & 3));
        } else {
            // fields that overlap byte b - nidx of the code stream
            const int bit0 = 8 * (b - nidx);
            const unsigned mask = (1u << bits) - 1u;
            v = 0;
            for (int m = bit0 / bits; m < k && m * bits < bit0 + 8; ++m) {
                const int sh = m * bits - bit0;
                const unsigned cde = (unsigned)codes[c * k + m] & mask;
                v |= sh >= 0 ? cde << sh : cde >> (-sh);
            }
        }
        out[o] = (unsigned char)v;
    }
}

// Record encoder, one thread per 32-bit word of the output: for records that are whole words
// with the code stream starting on a word (k a multiple of 8, record a multiple of 4 bytes) and
// 4-byte aligned `out` (and `codes` at 2 bits).  Same bytes as the byte-wise kernels above.
SL_DEV void pack_word(const uint16_t *idx, const uint8_t *codes, const float *values, int k, int bits, int wpr,
                      long long c0, int lw, unsigned magic, unsigned *out)
{
    const int cl = (int)__umulhi((unsigned)lw, magic);
    const long long c = c0 + cl;
    const int w = lw - cl * wpr, niw = 3 * k / 8;
    const uint16_t *ic = idx + c * k;
    unsigned v = 0;
    if (w < niw) {
        // the (up to four) 12-bit fields that overlap bits 32w .. 32w+31 of the index stream
        const int bit0 = 32 * w;
        int m = bit0 / 12;
#pragma unroll
        for (int q = 0; q < 4; ++q, ++m) {
            const int sh = 12 * m - bit0;
            if (m < k && sh < 32) {
                const unsigned x = (unsigned)ic[m] & 0xFFFu;
                v |= sh >= 0 ? x << sh : x >> (-sh);
            }
        }
    } else if (bits == 32) {
        v = __float_as_uint(values[c * k + (w - niw)]);
    } else if (bits == 2) {
        // sixteen codes, one per byte, from four aligned words
        const unsigned *cw = reinterpret_cast<const unsigned *>(codes + c * k) + 4 * (w - niw);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned x = cw[q];
            v |= ((x & 3u) | ((x >> 6) & 0xCu) | ((x >> 12) & 0x30u) | ((x >> 18) & 0xC0u)) << (8 * q);
        }
    } else {
        const int bit0 = 32 * (w - niw);
        const unsigned mask = (1u << bits) - 1u;
        const uint8_t *cc = codes + c * k;
        for (int m = bit0 / bits; m < k && m * bits < bit0 + 32; ++m) {
            const int sh = m * bits - bit0;
            const unsigned cde = (unsigned)cc[m] & mask;
            v |= sh >= 0 ? cde << sh : cde >> (-sh);
        }
    }
    out[c0 * wpr + lw] = v;
}

__global__ void __launch_bounds__(256)
k_pack_words(const uint16_t *idx, const uint8_t *codes, const float *values, long long n_chunks, int k, int bits,
             int wpr, int cpb, unsigned magic, unsigned *out)
{
    // a block encodes `cpb` consecutive chunks: their records are one run of cpb*wpr words, and a
    // word's chunk within the run is a multiplication away (magic = floor(2^32/wpr) + 1, exact
    // while word * wpr < 2^32)
    const long long c0 = (long long)blockIdx.x * cpb;
    const int nloc = (int)min((long long)cpb, n_chunks - c0) * wpr;
    for (int lw = threadIdx.x; lw < nloc; lw += blockDim.x)
        pack_word(idx, codes, values, k, bits, wpr, c0, lw, magic, out);
}


// The word-wise encoder serves the call if the record layout and the pointers allow it.
bool pack_words(const uint16_t *idx, const uint8_t *codes, const float *values, int64_t n_chunks, int k, int bits,
                unsigned char *out, hipStream_t st)
{
    const long long rec = sl_rec_bytes(k, bits);
    if ((k & 7) || (rec & 3) || ((uintptr_t)out & 3)) return false;
    if (bits == 2 && (((uintptr_t)codes & 3) || (k & 15))) return false;
    const int wpr = (int)(rec >> 2);
    int cpb = 4096 / wpr;                                     // about 16 words per thread
    cpb = cpb < 1 ? 1 : cpb > 64 ? 64 : cpb;
    const long long blocks = (n_chunks + cpb - 1) / cpb;
    if (blocks > 0x7FFFFFFFll) return false;                  // beyond one grid: the grid-stride kernel
    hipLaunchKernelGGL(k_pack_words, dim3((unsigned)blocks), dim3(256), 0, st, idx, codes, values,
                       (long long)n_chunks, k, bits, wpr, cpb, (unsigned)(0x100000000ull / (unsigned)wpr + 1),
                       reinterpret_cast<unsigned *>(out));
    return true;
}

}  // namespace

int slk_pack_bits(const uint16_t *idx, const uint8_t *codes, const float *values, int64_t n_chunks, int k,
                  int bits, unsigned char *out, hipStream_t st)
{
    const long long total = n_chunks * (long long)sl_rec_bytes(k, bits);
    if (total == 0) return SL_OK;
    long long blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (!pack_words(idx, codes, values, n_chunks, k, bits, out, st))
        hipLaunchKernelGGL(k_pack_bits, dim3((unsigned)blocks), dim3(256), 0, st, idx, codes, values,
                       (long long)n_chunks, k, bits, out);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    return SL_OK;
}

int slk_apply(const sl_plan *p, float *theta, float *mom, float mu, const void *const *payloads, int R,
              float lr, hipStream_t st)
{
    if (p->n_chunks == 0) return SL_OK;
    ApplyArgs A;
    A.desc = p->d_desc;
    A.theta = theta;
    A.mom = mom;
    A.mu = mu;
    A.neg_lr = -lr;
    A.inv_R = 1.0f / (float)R;
    A.R = R;
    A.k = p->k;
    A.bits = p->bits;
    A.hdr_bytes = p->hdr_bytes;
    A.rec_bytes = p->rec_bytes;
    const int rec_pad = ((p->rec_bytes + 3) & ~3) + p->hdr_bytes;
    // at most 16 KB of staged records; 4 KB on the eight-entry route (measured against 2, 8 and 16 KB:
    // more waves per compute unit outweigh the extra staging rounds), and whenever a record alone is large
    // ... and, four entries per lane, 2-bit records from k = 136 when there is much to decode (measured at
    // 16 workers: k = 160 0.90 -> 0.83 ms, k = 192 1.31 -> 0.86 ms; below 2048 entries per chunk the two-halves
    // route is as fast or faster)
    const bool octets = (p->k & 7) == 0 &&
                        (p->k >= SL_APPLY_OCTETS_FROM ||
                         (p->bits == 2 && p->k >= SL_APPLY_QUADS_FROM && (long long)R * p->k >= SL_APPLY_QUADS_ENTRIES));
    int batch = (rec_pad > 1024 || octets ? SL_APPLY_BIG_STAGE : 16384) / rec_pad;
    if (batch < 1) batch = 1;
    if (batch > R) batch = R;
    A.batch = batch;
    A.magic_src = (unsigned)(0x100000000ull / (unsigned)(rec_pad >> 2) + 1);
#ifndef SL_APPLY_QUADS_BELOW
#define SL_APPLY_QUADS_BELOW 257
#endif
    A.quads = octets && p->bits == 2 && p->k < SL_APPLY_QUADS_BELOW;
    for (int r = 0; r < SL_MAX_WORKERS; ++r)
        A.payload[r] = r < R ? static_cast<const unsigned char *>(payloads[r]) : nullptr;
    A.n_chunks = p->n_chunks;
    // (not when the staged records themselves are the larger part of the LDS: nothing would be gained)
    // (not on the eight-entry route: with 4 KB staged at a time the halves would fetch every record twice)
    const bool halves = (long long)R * p->k >= SL_APPLY_HALVES_FROM && (size_t)batch * rec_pad <= 8192 && !octets;
    const size_t acc_bytes = SL_CHUNK * sizeof(float) / (halves ? 2 : 1);
    A.lds_per_wave = (int)((acc_bytes + (size_t)batch * rec_pad + 15) & ~(size_t)15);
    int wpb = 4;
    while (wpb > 1 && (size_t)A.lds_per_wave * wpb > (size_t)p->max_lds) wpb >>= 1;
    const size_t lds = (size_t)A.lds_per_wave * wpb;
    const bool two = p->bits == 2;
    typedef void (*kernel_t)(ApplyArgs);
    const int route = (!halves && p->k <= 128) ? 0 : !octets ? 1 : 2;
#define SL_APPLY_ROUTES(TWO, NEST) \
    {k_apply<TWO, NEST, 1, 0>, k_apply<TWO, NEST, 1, 1>, k_apply<TWO, NEST, 1, 2>, k_apply<TWO, NEST, 2, 1>}
    static const kernel_t table[2][2][4] = {{SL_APPLY_ROUTES(false, false), SL_APPLY_ROUTES(false, true)},
                                            {SL_APPLY_ROUTES(true, false), SL_APPLY_ROUTES(true, true)}};
#undef SL_APPLY_ROUTES
    const kernel_t fn = table[two ? 1 : 0][mom ? 1 : 0][halves ? 3 : route];   // (two halves: entry by entry only)
    if (lds > 65536) {
        hipError_t aerr = hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (aerr != hipSuccess) {
            sl_note_hip_error(aerr);
            return SL_ERR_HIP;
        }
    }
    const dim3 grid((unsigned)((p->n_chunks + wpb - 1) / wpb)), block(64 * wpb);
    hipLaunchKernelGGL(fn, grid, block, lds, st, A);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    return SL_OK;
}

int slk_validate(const sl_plan *p, const unsigned char *payload, int *flag, hipStream_t st)
{
    hipError_t err = hipMemsetAsync(flag, 0, sizeof(int), st);
    if (err == hipSuccess && p->n_chunks > 0) {
        hipLaunchKernelGGL(k_validate, dim3((unsigned)((p->n_chunks + 3) / 4)), dim3(256), 0, st, p->d_desc,
                           (long long)p->n_chunks, p->k, payload, flag);
        err = hipGetLastError();
    }
    int host = 0;
    if (err == hipSuccess) err = hipMemcpyAsync(&host, flag, sizeof(int), hipMemcpyDeviceToHost, st);
    if (err == hipSuccess) err = hipStreamSynchronize(st);
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    return host ? SL_ERR_BAD_PAYLOAD : SL_OK;
}

int slk_pack(const uint16_t *idx, const uint8_t *codes, int64_t n_chunks, int k, unsigned char *out,
             hipStream_t st)
{
    const long long total = n_chunks * ((long long)7 * k / 4);
    if (total == 0) return SL_OK;
    long long blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (!pack_words(idx, codes, nullptr, n_chunks, k, 2, out, st))
        hipLaunchKernelGGL(k_pack, dim3((unsigned)blocks), dim3(256), 0, st, idx, codes,
                       (long long)n_chunks, k, out);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    return SL_OK;
}
