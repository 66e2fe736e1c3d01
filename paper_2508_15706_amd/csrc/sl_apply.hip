// sl_decompress_avg_apply: dequantise R workers' sparse payloads, average and
// take the outer SGD step in one pass over theta (Algorithm 1, "Aggregate +
// Outer Update"; Eq. (2) lines 3-4), and the stand-alone record encoder
// sl_pack_indices (12-bit index fields + 2-bit codes).
//
// One wavefront owns one chunk.  The dense average never exists in HBM: the
// chunk's fp32 accumulators live in LDS (one half of the chunk at a time, 8 KB),
// the R records (7k/4 bytes each) are staged into LDS with coalesced loads, entries of one worker are
// distinct positions so they are added without conflicts, workers are added in
// the order r = 0..R-1, and theta streams through registers once
// (8 bytes per element of HBM traffic plus R*7k/4 bytes per chunk).
#include "sl_device.h"
#include "sl_internal.h"

namespace {

// When there is much to decode per chunk (R*k entries), the chunk is aggregated
// in NH = 2 halves of 32 rows (local indices below / from 2048): 8 KB of
// accumulators per wave instead of 16, so that twice as many waves - and twice
// as many bytes of theta in flight - fit a compute unit while the decode runs.
// With little to decode one pass (NH = 1) is slightly faster.
constexpr int APPLY_HALVES_FROM = 768;       // R*k from which two halves pay (measured)

struct ApplyArgs {
    const SlChunkDesc *desc;
    float *theta;
    float *mom;              // global outer momentum buffer (Nesterov variant), else null
    float mu;
    float neg_lr, inv_R;
    int R, k;
    int bits, hdr_bytes, rec_bytes;   // value width and the sizes that follow from it
    int batch;               // records staged per round
    int lds_per_wave;
    long long n_chunks;
    const unsigned char *payload[SL_MAX_WORKERS];
};

// One wave per chunk, several independent waves (adjacent chunks) per workgroup.
// TWO_BIT: the 2-bit format with its four-entry table kept in registers;
// otherwise any width (table of 2^bits entries read from LDS, or fp32 values).
// NESTEROV: DiLoCo's global outer momentum on top of the aggregate (Eq. (1);
// appendix algorithm "Outer step for DiLoCo+Top-k[+EF]"): m <- mu*m + avg,
// d <- avg + mu*m, theta <- theta - lr*d at every element of the chunk.
template <bool TWO_BIT, bool NESTEROV, int NH>
__global__ void __launch_bounds__(256) k_apply(ApplyArgs A)
{
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

    // Word w of a batch's staging area: worker r = w / wpr_src, word q of (LUT, record)
    const bool word_path = (rec_bytes & 3) == 0;
    const int wpr_src = hdr_words + (rec_bytes >> 2);  // words per worker: LUT + record
    const int wpr_dst = rec_pad >> 2;
    auto src_word = [&](int r, int q) -> unsigned {
        const unsigned char *p = A.payload[r];
        return q < hdr_words ? reinterpret_cast<const unsigned *>(p + lut_off)[q]
                             : reinterpret_cast<const unsigned *>(p + rec_off)[q - hdr_words];
    };
    // The first 64*PF words of the first batch (all of it for R*(16 + 7k/4) <= 2 KB:
    // R = 8 up to k = 128, R = 16 up to k = 64) are fetched into registers BEFORE the
    // theta loads: loads complete in order, so the decode below then waits for these
    // few words only and runs while the chunk's 16 KB of theta are still in flight.
    constexpr int PF = TWO_BIT ? 8 : 12;   // wider records at other widths: 3 KB
    unsigned pf[PF];
    const int nb0 = min(A.batch, A.R);
    if (word_path) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int w = lane + 64 * u;
            pf[u] = 0;
            if (w < nb0 * wpr_src) {
                const int r = w / wpr_src;
                pf[u] = src_word(r, w - r * wpr_src);
            }
        }
    }

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
                if (word_path) {
                    int w0 = lane;
                    if (r0 == 0 && h == 0) {
#pragma unroll
                        for (int u = 0; u < PF; ++u) {
                            const int w = lane + 64 * u;
                            if (w < nb * wpr_src) {
                                const int r = w / wpr_src;
                                reinterpret_cast<unsigned *>(stage)[r * wpr_dst + (w - r * wpr_src)] = pf[u];
                            }
                        }
                        w0 = lane + 64 * PF;
                    }
                    for (int w = w0; w < nb * wpr_src; w += 64) {
                        const int r = w / wpr_src, q = w - r * wpr_src;
                        reinterpret_cast<unsigned *>(stage)[r * wpr_dst + q] = src_word(r0 + r, q);
                    }
                } else {
                    for (int w = lane; w < nb * hdr_words; w += 64) {    // the tensor's LUT of each worker
                        const int r = w / hdr_words, q = w - r * hdr_words;
                        reinterpret_cast<unsigned *>(stage)[r * wpr_dst + q] =
                            reinterpret_cast<const unsigned *>(A.payload[r0 + r] + lut_off)[q];
                    }
                    for (int b = lane; b < nb * rec_bytes; b += 64) {
                        const int r = b / rec_bytes, q = b - r * rec_bytes;
                        stage[r * rec_pad + hdr + q] = A.payload[r0 + r][rec_off + q];
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
            if (NH == 1 && k <= 128) {
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
                                    acc[j & (ACC_FLOATS - 1)] = acc[j & (ACC_FLOATS - 1)] + qq[u][s2];
                            }
                            sl_wave_sync();   // worker r is complete before worker r+1 is added
                        }
                    }
                }
            } else {
                for (int r = 0; r < nb; ++r) {
                    for (int m = lane; m < k; m += 64) {
                        unsigned j;
                        float q;
                        decode(r, m, j, q);
                        if (NH == 1 || (int)(j >> 11) == h)         // this half's entries
                            acc[j & (ACC_FLOATS - 1)] = acc[j & (ACC_FLOATS - 1)] + q;
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
            for (int i8 = 0; i8 < ROWS4; ++i8) {
                const int row = 4 * (ROWS4 * h + i8) + lr;
                const int lim = row < rows - 1 ? cols : (row == rows - 1 ? last_cols : 0);
                const unsigned o0 = row * stride + lc;
                if (lc + 3 < lim) {
                    // all four columns inside: one 16-byte access per stream (rows need no alignment)
                    const float4 a = reinterpret_cast<const float4 *>(acc)[i8 * 64 + lane];
                    sl_f4 g;
                    g.x = a.x * A.inv_R, g.y = a.y * A.inv_R, g.z = a.z * A.inv_R, g.w = a.w * A.inv_R;
                    if constexpr (NESTEROV) {
                        sl_f4 m = sl_load_stream_u(mc + o0);
                        m.x = fmaf(A.mu, m.x, g.x), m.y = fmaf(A.mu, m.y, g.y);
                        m.z = fmaf(A.mu, m.z, g.z), m.w = fmaf(A.mu, m.w, g.w);
                        sl_store_stream_u(mc + o0, m);
                        g.x = fmaf(A.mu, m.x, g.x), g.y = fmaf(A.mu, m.y, g.y);
                        g.z = fmaf(A.mu, m.z, g.z), g.w = fmaf(A.mu, m.w, g.w);
                    }
                    sl_f4 v = sl_load_stream_u(tc + o0);
                    v.x = fmaf(A.neg_lr, g.x, v.x), v.y = fmaf(A.neg_lr, g.y, v.y);
                    v.z = fmaf(A.neg_lr, g.z, v.z), v.w = fmaf(A.neg_lr, g.w, v.w);
                    sl_store_stream_u(tc + o0, v);
                } else {
                    for (int cc = 0; cc < 4; ++cc) {
                        if (lc + cc < lim) {
                            const unsigned o = o0 + cc;
                            float g = acc[256 * i8 + 4 * lane + cc] * A.inv_R;
                            if constexpr (NESTEROV) {
                                const float m = fmaf(A.mu, mc[o], g);
                                mc[o] = m;
                                g = fmaf(A.mu, m, g);
                            }
                            tc[o] = fmaf(A.neg_lr, g, tc[o]);
                        }
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

}  // namespace

int slk_pack_bits(const uint16_t *idx, const uint8_t *codes, const float *values, int64_t n_chunks, int k,
                  int bits, unsigned char *out, hipStream_t st)
{
    const long long total = n_chunks * (long long)sl_rec_bytes(k, bits);
    if (total == 0) return SL_OK;
    long long blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
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
    // at most 16 KB of staged records; 4 KB when a record alone is large (k >= 1024), so that the
    // accumulators are not crowded out of the LDS
    int batch = (rec_pad > 1024 ? 4096 : 16384) / rec_pad;
    if (batch < 1) batch = 1;
    if (batch > R) batch = R;
    A.batch = batch;
    for (int r = 0; r < SL_MAX_WORKERS; ++r)
        A.payload[r] = r < R ? static_cast<const unsigned char *>(payloads[r]) : nullptr;
    A.n_chunks = p->n_chunks;
    // (not when the staged records themselves are the larger part of the LDS: nothing would be gained)
    const bool halves = (long long)R * p->k >= APPLY_HALVES_FROM && (size_t)batch * rec_pad <= 8192;
    const size_t acc_bytes = SL_CHUNK * sizeof(float) / (halves ? 2 : 1);
    A.lds_per_wave = (int)((acc_bytes + (size_t)batch * rec_pad + 15) & ~(size_t)15);
    int wpb = 4;
    while (wpb > 1 && (size_t)A.lds_per_wave * wpb > (size_t)p->max_lds) wpb >>= 1;
    const size_t lds = (size_t)A.lds_per_wave * wpb;
    const bool two = p->bits == 2;
    typedef void (*kernel_t)(ApplyArgs);
    static const kernel_t table[2][2][2] = {
        {{k_apply<false, false, 1>, k_apply<false, false, 2>}, {k_apply<false, true, 1>, k_apply<false, true, 2>}},
        {{k_apply<true, false, 1>, k_apply<true, false, 2>}, {k_apply<true, true, 1>, k_apply<true, true, 2>}}};
    const kernel_t fn = table[two ? 1 : 0][mom ? 1 : 0][halves ? 1 : 0];
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
    hipLaunchKernelGGL(k_pack, dim3((unsigned)blocks), dim3(256), 0, st, idx, codes,
                       (long long)n_chunks, k, out);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    return SL_OK;
}
