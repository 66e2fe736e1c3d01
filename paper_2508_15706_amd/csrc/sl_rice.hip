// Index coder: transcodes a payload between the plain wire format (12-bit
// indices) and a Rice-coded format (appendix "Compression of indices in Top-k":
// the paper compresses the indices with "sub-chunking and Rice coding" and
// reports 8.9 / 6.6 / 5.6 bits per index for k = 32 / 128 / 256; the algorithm is
// not described, the format below is this library's own).
//
// Coded format.  An ascending index list is coded as gaps g_0 = idx_0,
// g_i = idx_i - idx_(i-1) - 1, each as a Rice code with parameter
// b = floor(log2(2839 / k)) (0 when 2839 / k < 1; 2839 = floor(4096 ln 2)):
// (g >> b) one-bits, a zero bit, the b low bits of g LSB first; bits fill bytes
// LSB first.  A chunk is its k gap codes followed by its k 2-bit codes.  The
// chunks of a GROUP of 8 follow each other without padding, a group starts on
// a 4-byte boundary.  Tensor block (16-byte aligned): float LUT[4]; uint32
// goff[n_groups] = byte offset of each group from the block start; the
// streams; zero padding to 16.  Buffer: "SLRICE01", uint64 total bytes, uint64
// tensor_off[n_tensors], zero padding to 16, the blocks.  At another value
// width (1, 3, 4 bits, or 32 = unquantized) the table has 2^bits floats padded
// to 16 bytes (none at 32) and a chunk's gap codes are followed by its k value
// fields of that width, as they stand in the plain record.
//
// One lane codes or decodes one group sequentially (a group is the unit that
// cannot be split); sizes are found first, then two small scans place the
// groups and the tensor blocks, then the streams are written.
#include "sl_device.h"
#include "sl_internal.h"

int sl_rice_param(int k)
{
    const int q = 2839 / k;
    int b = 0;
    while ((2 << b) <= q) ++b;
    return q < 1 ? 0 : b;
}

namespace {

// Sequential reader of bit fields from a byte- or word-addressed stream (the encoder's reader of
// plain records: all lanes consume the same number of bits per call, so they load together).
template <bool WORDS>
struct BitReader {
    const unsigned char *p, *end;
    unsigned long long acc = 0;
    int n = 0;
    SL_DEV BitReader(const unsigned char *start, const unsigned char *limit) : p(start), end(limit) {}
    SL_DEV void refill()
    {
        if (WORDS) {
            const unsigned w = p + 4 <= end ? *reinterpret_cast<const unsigned *>(p) : 0u;
            acc |= (unsigned long long)w << n;
            p += 4, n += 32;
        } else {
            const unsigned w = p < end ? *p : 0u;
            acc |= (unsigned long long)w << n;
            p += 1, n += 8;
        }
    }
    SL_DEV unsigned get(int bits)            // bits <= 32
    {
        while (n < bits) refill();
        const unsigned v = bits == 32 ? (unsigned)acc : (unsigned)acc & ((1u << bits) - 1u);
        acc >>= bits, n -= bits;
        return v;
    }
    SL_DEV unsigned unary()                  // number of one-bits before the next zero bit
    {
        unsigned q = 0;
        for (;;) {
            if (n == 0) refill();
            const unsigned long long inv = ~acc;
            const int t = inv ? __ffsll((long long)inv) - 1 : 64;
            if (t >= n) {                    // every buffered bit is a one
                q += n;
                acc = 0, n = 0;
                if (q > 8192) return q;      // malformed input: stop
            } else {
                q += t;
                acc >>= (t + 1), n -= (t + 1);
                return q;
            }
        }
    }
};

// The decoder's reader.  The lanes of a wave decode different streams in lockstep (same k, same
// loops) but sit at different bit positions, so with a reader that loads on demand some lane
// loads on nearly every entry, and the wait that follows is for the whole wave.  Here every
// lane keeps a window of W words of its stream in LDS (word-interleaved over the lanes) and all
// lanes top their windows up together at fixed points of the loops; in between they read LDS
// only.  W covers the most bits that can be consumed between two such points (see
// rice_window_words); a malformed stream that consumes more reads stale words of the window -
// garbage, as beyond the end of the input, but always inside the window.
struct WinReader {
    const unsigned char *src, *end;          // next word of the stream to load; end of the input
    unsigned *win;                           // this wave's windows, word w of lane l at [w * 64 + l]
    unsigned wmask;                          // W - 1, W a power of two
    int lane;
    unsigned fill = 0, rdw = 0;              // words loaded / handed out so far
    unsigned long long acc = 0;
    int n = 0;
    SL_DEV WinReader(const unsigned char *start, const unsigned char *limit, unsigned *w, int W, int l)
        : src(start), end(limit), win(w), wmask((unsigned)W - 1u), lane(l)
    {
        top_up();
    }
    SL_DEV void top_up()                     // called by the lanes of a wave together
    {
        const unsigned room = (wmask + 1u) - (fill - rdw);
        for (unsigned j0 = 0; sl_ballot(j0 < room) != 0ull; j0 += 8) {
            unsigned v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const unsigned char *p = src + 4ull * (j0 + u);
                v[u] = (j0 + u < room && p + 4 <= end) ? *reinterpret_cast<const unsigned *>(p) : 0u;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (j0 + u < room) win[((fill + j0 + u) & wmask) * 64u + lane] = v[u];
        }
        src += 4ull * room;
        fill += room;
    }
    SL_DEV void refill()
    {
        const unsigned w = win[(rdw & wmask) * 64u + lane];
        ++rdw;
        acc |= (unsigned long long)w << n;
        n += 32;
    }
    SL_DEV unsigned get(int bits)            // bits <= 32
    {
        while (n < bits) refill();
        const unsigned v = bits == 32 ? (unsigned)acc : (unsigned)acc & ((1u << bits) - 1u);
        acc >>= bits, n -= bits;
        return v;
    }
    SL_DEV unsigned unary()                  // number of one-bits before the next zero bit
    {
        unsigned q = 0;
        for (;;) {
            if (n == 0) refill();
            const unsigned long long inv = ~acc;
            const int t = inv ? __ffsll((long long)inv) - 1 : 64;
            if (t >= n) {                    // every buffered bit is a one
                q += n;
                acc = 0, n = 0;
                if (q > 8192) return q;      // malformed input: stop
            } else {
                q += t;
                acc >>= (t + 1), n -= (t + 1);
                return q;
            }
        }
    }
};

// Sequential writer; COUNT = only count the bits.
template <bool COUNT, bool WORDS>
struct BitWriter {
    unsigned char *p;
    unsigned long long acc = 0;
    int n = 0;
    long long total = 0;
    SL_DEV explicit BitWriter(unsigned char *start) : p(start) {}
    SL_DEV void put(unsigned v, int bits)    // bits <= 32, v < 2^bits
    {
        total += bits;
        if (COUNT) return;
        acc |= (unsigned long long)v << n;
        n += bits;
        if (WORDS) {
            if (n >= 32) {
                *reinterpret_cast<unsigned *>(p) = (unsigned)acc;
                p += 4, acc >>= 32, n -= 32;
            }
        } else {
            while (n >= 8) {
                *p++ = (unsigned char)acc;
                acc >>= 8, n -= 8;
            }
        }
    }
    SL_DEV void flush_word()                 // pad with zero bits to a 4-byte boundary
    {
        const int pad = (int)((32 - (total & 31)) & 31);
        if (pad) put(0u, pad);
    }
};

struct RiceArgs {
    const SlChunkDesc *desc;
    const SlTensorDev *tensors;
    const SlGroup *groups;
    long long n_groups;
    int n_tensors;
    int k, b;
    int bits, hdr_bytes, rec_bytes;   // value width of the payload and the sizes that follow from it
    unsigned *gsize;               // [n_groups] coded bytes of each group
    unsigned *goff;                // [n_groups] byte offset of each group in its block
    unsigned long long *tbytes;    // [n_tensors] bytes of each tensor block
};

// Codes the chunks of group G from the plain payload.  COUNT: returns the
// coded bytes only.  Otherwise writes the stream at `dst` (4-byte aligned).
template <bool COUNT, bool WORDS>
SL_DEV unsigned code_group(const RiceArgs &A, long long G, const unsigned char *payload,
                           unsigned char *dst)
{
    const SlGroup g = A.groups[G];
    const SlTensorDev td = A.tensors[g.tensor];
    const int k = A.k, b = A.b;
    const long long rec = A.rec_bytes;
    const long long c0 = (long long)g.local_group * SL_RICE_GROUP;
    const int nc = (int)min((long long)SL_RICE_GROUP, td.n_chunks - c0);
    BitWriter<COUNT, true> w(dst);
    for (int i = 0; i < nc; ++i) {
        const unsigned char *r = payload + td.pay_off + A.hdr_bytes + (c0 + i) * rec;
        BitReader<WORDS> rd(r, r + rec);
        int prev = -1;
        for (int m = 0; m < k; ++m) {
            const int idx = (int)rd.get(12);
            unsigned gap = (unsigned)(idx - prev - 1);
            prev = idx;
            unsigned q = gap >> b;
            const unsigned rem = gap & ((1u << b) - 1u);
            if (q + 1u + (unsigned)b <= 32u) {
                // the usual case in one piece: q one-bits, the zero bit, the remainder
                w.put(((1u << q) - 1u) | (rem << (q + 1u)), (int)q + 1 + b);
            } else {
                while (q >= 32) {
                    w.put(0xFFFFFFFFu, 32);
                    q -= 32;
                }
                if (q) w.put((1u << q) - 1u, (int)q);
                w.put(rem << 1, b + 1);                           // the zero bit, then the remainder
            }
        }
        // the k value fields as they stand in the record (k * bits is a multiple of 8)
        int left = k * A.bits;
        const int piece = WORDS ? 32 : 8;
        for (; left >= piece; left -= piece) w.put(rd.get(piece), piece);
        if (left) w.put(rd.get(left), left);
    }
    w.flush_word();
    return (unsigned)(w.total >> 3);
}

template <bool WORDS>
__global__ void __launch_bounds__(64) k_rice_sizes(RiceArgs A, const unsigned char *payload)
{
    const long long G = (long long)blockIdx.x * 64 + threadIdx.x;
    if (G >= A.n_groups) return;
    A.gsize[G] = code_group<true, WORDS>(A, G, payload, nullptr);
}

// One workgroup per tensor: exclusive scan of its groups' sizes.
__global__ void __launch_bounds__(256) k_rice_scan(RiceArgs A)
{
    __shared__ unsigned long long wsum[4];
    __shared__ unsigned long long carry;
    const SlTensorDev td = A.tensors[blockIdx.x];
    const long long ng = (td.n_chunks + SL_RICE_GROUP - 1) / SL_RICE_GROUP;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = (unsigned long long)A.hdr_bytes + 4ull * (unsigned long long)ng;
    __syncthreads();
    for (long long base = 0; base < ng; base += 256) {
        const long long i = base + tid;
        const unsigned long long v = i < ng ? A.gsize[td.group0 + i] : 0ull;
        unsigned long long incl = v;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const unsigned long long up = __shfl_up(incl, s);
            if (lane >= s) incl += up;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        unsigned long long before = carry;
        for (int q = 0; q < wave; ++q) before += wsum[q];
        if (i < ng) A.goff[td.group0 + i] = (unsigned)(before + incl - v);
        __syncthreads();
        if (tid == 255) carry = before + incl;
        __syncthreads();
    }
    if (tid == 0) A.tbytes[blockIdx.x] = (carry + 15ull) & ~15ull;
}

// Header: magic, total, tensor offsets (one wave scans the tensor blocks' sizes, 64 at a time).
__global__ void __launch_bounds__(64) k_rice_header(RiceArgs A, unsigned char *out)
{
    const int lane = threadIdx.x;
    unsigned long long *h = reinterpret_cast<unsigned long long *>(out);
    unsigned long long pos = (16ull + 8ull * (unsigned long long)A.n_tensors + 15ull) & ~15ull;
    for (int base = 0; base < A.n_tensors; base += 64) {
        const int t = base + lane;
        const unsigned long long v = t < A.n_tensors ? A.tbytes[t] : 0ull;
        unsigned long long incl = v;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const unsigned long long up = __shfl_up(incl, s);
            if (lane >= s) incl += up;
        }
        if (t < A.n_tensors) h[2 + t] = pos + incl - v;
        pos += __shfl(incl, 63);
    }
    if (lane == 0) {
        if ((A.n_tensors & 1)) h[2 + A.n_tensors] = 0ull;      // padding of the header to 16 bytes
        h[0] = 0x3130454349524C53ull;                          // "SLRICE01", little endian
        h[1] = pos;
    }
}

template <bool WORDS>
__global__ void __launch_bounds__(64) k_rice_encode(RiceArgs A, const unsigned char *payload,
                                                    unsigned char *out)
{
    const long long G = (long long)blockIdx.x * 64 + threadIdx.x;
    if (G >= A.n_groups) return;
    const SlGroup g = A.groups[G];
    const SlTensorDev td = A.tensors[g.tensor];
    unsigned char *blk = out + reinterpret_cast<const unsigned long long *>(out)[2 + g.tensor];
    const unsigned off = A.goff[G];
    reinterpret_cast<unsigned *>(blk + A.hdr_bytes)[g.local_group] = off;
    const unsigned bytes = code_group<false, WORDS>(A, G, payload, blk + off);
    if (g.local_group == 0)                                    // the look-up table (a multiple of 16 bytes)
        for (int q = 0; q < A.hdr_bytes; q += 16)
            *reinterpret_cast<float4 *>(blk + q) = *reinterpret_cast<const float4 *>(payload + td.pay_off + q);
    const long long ng = (td.n_chunks + SL_RICE_GROUP - 1) / SL_RICE_GROUP;
    if (g.local_group == ng - 1)                               // zero padding of the block
        for (unsigned long long q = off + bytes; q < A.tbytes[g.tensor]; q += 4)
            *reinterpret_cast<unsigned *>(blk + q) = 0u;
}

// Entries between two top-ups of the decoder's windows, and the window that covers them: the
// gaps of `epr` entries of one chunk take at most epr * (1 + b) bits plus 4096 >> b one-bits
// (the unary parts of a chunk add up to at most 4095 >> b), up to 64 consumed bits still sit in
// the reader's register, and a word may be half used on either side.
constexpr int RICE_EPR = 16;
static int rice_window_words(int b)
{
    const int bits = RICE_EPR * (1 + b) + (4096 >> b);
    int need = (bits + 31) / 32 + 4, W = 16;      // (at least 16: the value fields are copied 8 words at a time)
    while (W < need) W <<= 1;
    return W;
}

template <bool WORDS>
__global__ void __launch_bounds__(64) k_rice_decode(RiceArgs A, const unsigned char *in,
                                                    unsigned long long in_bytes, unsigned char *payload, int W)
{
    extern __shared__ unsigned rice_win[];
    const int lane = threadIdx.x;
    const long long G = (long long)blockIdx.x * 64 + lane;
    // (a lane beyond the last group stays in the wave: the windows are topped up by all lanes together)
    const bool live = G < A.n_groups;
    const SlGroup g = live ? A.groups[G] : SlGroup{0, 0};
    const SlTensorDev td = A.tensors[g.tensor];
    const int k = A.k, b = A.b, hdr = A.hdr_bytes;
    const long long rec = A.rec_bytes;
    const unsigned char *end = in + in_bytes;
    unsigned long long toff = reinterpret_cast<const unsigned long long *>(in)[2 + g.tensor];
    if (toff > in_bytes) toff = in_bytes;
    const unsigned char *blk = in + toff;
    unsigned long long off = in_bytes;                         // beyond the end: reads as zeros
    if (live && blk + hdr + 4ull * (g.local_group + 1) <= end)
        off = toff + reinterpret_cast<const unsigned *>(blk + hdr)[g.local_group];
    if (off > in_bytes) off = in_bytes;
    WinReader rd(in + (off & ~3ull), end, rice_win, W, lane);
    const long long c0 = (long long)g.local_group * SL_RICE_GROUP;
    const int nc = live ? (int)min((long long)SL_RICE_GROUP, td.n_chunks - c0) : 0;
    for (int i = 0; i < nc; ++i) {
        unsigned char *r = payload + td.pay_off + hdr + (c0 + i) * rec;
        BitWriter<false, WORDS> w(r);
        int prev = -1;
        for (int m = 0; m < k; ++m) {
            if ((m & (RICE_EPR - 1)) == 0) rd.top_up();
            // Common case in straight-line code: with 32 bits buffered, a unary part and a
            // remainder that end inside them are taken with one count of trailing ones and one
            // shift; a longer code goes through the general calls.  (The lanes of a wave run
            // this loop as one instruction stream, and there is less than one wave per SIMD:
            // the length of that stream is what the decoder's time is - 0.27 -> 0.16 ms at
            // configuration 4.  Collecting the records in LDS and writing them out 64 words
            // at a time instead of one word per lane gained 2 % and was left out.)
            if (rd.n < 32) rd.refill();
            const unsigned low = (unsigned)rd.acc;
            const int t = __ffs((int)~low) - 1;                 // one-bits before the first zero (-1: 32 ones)
            unsigned gap;
            if (t >= 0 && t + 1 + b <= 32) {
                gap = ((unsigned)t << b) | (unsigned)((rd.acc >> (t + 1)) & ((1ull << b) - 1ull));
                rd.acc >>= (t + 1 + b), rd.n -= (t + 1 + b);
            } else {
                const unsigned q = rd.unary();
                gap = (q << b) | rd.get(b);
            }
            int idx = prev + 1 + (int)gap;
            if (idx > 4095 || idx < 0) idx = 4095;             // malformed input stays in range
            prev = idx;
            w.put((unsigned)idx, 12);
        }
        int left = k * A.bits;
        const int piece = WORDS ? 32 : 8;
        for (int cnt = 0; left >= piece; left -= piece, ++cnt) {
            if ((cnt & (WORDS ? 7 : 31)) == 0) rd.top_up();    // every 8 words of value fields
            w.put(rd.get(piece), piece);
        }
        if (left) w.put(rd.get(left), left);
    }
    if (!live) return;
    if (g.local_group == 0) {
        for (int q = 0; q < hdr; q += 16) {
            float4 lut = make_float4(0.f, 0.f, 0.f, 0.f);
            if (blk + q + 16 <= end) lut = *reinterpret_cast<const float4 *>(blk + q);
            *reinterpret_cast<float4 *>(payload + td.pay_off + q) = lut;
        }
    }
    const long long ng = (td.n_chunks + SL_RICE_GROUP - 1) / SL_RICE_GROUP;
    if (g.local_group == ng - 1)                               // padding of the plain tensor block
        for (long long q = hdr + td.n_chunks * rec; q < td.block_bytes; ++q) payload[td.pay_off + q] = 0;
}

int launched()
{
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    return SL_OK;
}

RiceArgs make_args(const sl_plan *p, unsigned char *ws)
{
    RiceArgs A;
    A.desc = p->d_desc;
    A.tensors = p->d_tensors;
    A.groups = p->d_groups;
    A.n_groups = p->n_groups;
    A.n_tensors = p->n_tensors;
    A.k = p->k;
    A.b = sl_rice_param(p->k);
    A.bits = p->bits;
    A.hdr_bytes = p->hdr_bytes;
    A.rec_bytes = p->rec_bytes;
    const size_t sec = ((size_t)p->n_groups * 4 + 255) & ~(size_t)255;
    A.gsize = ws ? reinterpret_cast<unsigned *>(ws) : nullptr;
    A.goff = ws ? reinterpret_cast<unsigned *>(ws + sec) : nullptr;
    A.tbytes = ws ? reinterpret_cast<unsigned long long *>(ws + 2 * sec) : nullptr;
    return A;
}

}  // namespace

int slk_rice_encode(const sl_plan *p, const unsigned char *payload, unsigned char *out,
                    unsigned char *ws, hipStream_t st)
{
    const RiceArgs A = make_args(p, ws);
    const bool words = (p->rec_bytes & 3) == 0 && ((3 * p->k / 2) & 3) == 0;   // records and their value runs are 4-byte aligned
    const unsigned nblk = (unsigned)((p->n_groups + 63) / 64);
    int rc;
    if (p->n_groups > 0) {
        if (words) hipLaunchKernelGGL(k_rice_sizes<true>, dim3(nblk), dim3(64), 0, st, A, payload);
        else hipLaunchKernelGGL(k_rice_sizes<false>, dim3(nblk), dim3(64), 0, st, A, payload);
        if ((rc = launched())) return rc;
        hipLaunchKernelGGL(k_rice_scan, dim3(p->n_tensors), dim3(256), 0, st, A);
        if ((rc = launched())) return rc;
    }
    hipLaunchKernelGGL(k_rice_header, dim3(1), dim3(64), 0, st, A, out);
    if ((rc = launched())) return rc;
    if (p->n_groups > 0) {
        if (words) hipLaunchKernelGGL(k_rice_encode<true>, dim3(nblk), dim3(64), 0, st, A, payload, out);
        else hipLaunchKernelGGL(k_rice_encode<false>, dim3(nblk), dim3(64), 0, st, A, payload, out);
        if ((rc = launched())) return rc;
    }
    return SL_OK;
}

int slk_rice_decode(const sl_plan *p, const unsigned char *in, size_t in_bytes, unsigned char *payload,
                    hipStream_t st)
{
    if (p->n_groups == 0) return SL_OK;
    const RiceArgs A = make_args(p, nullptr);
    const bool words = (p->rec_bytes & 3) == 0 && ((3 * p->k / 2) & 3) == 0;
    const unsigned nblk = (unsigned)((p->n_groups + 63) / 64);
    const int W = rice_window_words(A.b);                      // <= 256 words: 64 KB of LDS at most
    const size_t lds = (size_t)W * 64 * sizeof(unsigned);
    if (words)
        hipLaunchKernelGGL(k_rice_decode<true>, dim3(nblk), dim3(64), lds, st, A, in,
                           (unsigned long long)in_bytes, payload, W);
    else
        hipLaunchKernelGGL(k_rice_decode<false>, dim3(nblk), dim3(64), lds, st, A, in,
                           (unsigned long long)in_bytes, payload, W);
    return launched();
}
