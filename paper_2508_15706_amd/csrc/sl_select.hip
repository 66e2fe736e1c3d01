// Kernel A of sl_compress: error-feedback accumulate fused with the chunk-wise
// Top-k selection (Eq. (2) line 1 and the Top-k of line 2; Section 3.3 last
// paragraph for the chunking).
//
// One 64-lane wavefront owns one 4096-element chunk, 64 elements per lane in
// registers.  HBM traffic per chunk: 16 KB of e and 16 KB of delta read once,
// 16 KB of e written once, plus 3k/2 bytes of packed indices, 4k bytes of
// selected values and 16 bytes of partial sums.
//
// Register r = 4*i + cc of lane l holds local index j = 256*i + 4*l + cc, i.e.
// the lane's i-th 16-byte load.  With rows of 64 elements this is row
// 4*i + l/16, columns 4*(l%16) .. +3 for both chunk layouts.
//
// Selection = exact k-th largest magnitude key T by bitwise bisection with
// wave ballots as the counting primitive, made cheap by pruning first:
//   1. every lane keeps the maxima of GPL groups of its registers; the k-th
//      largest of those 64*GPL maxima is a lower bound L of T (there are k
//      distinct elements >= L);
//   2. keys >= L (typically ~1.4k of them) are compacted into LDS and T is
//      bisected over that short list only;
//   3. one ordered compaction over the registers emits the selected entries in
//      ascending local index; ties at T go to the lowest indices.
// If the candidate list overflows (massive ties) or k is large, T is bisected
// over the registers directly - slower, same result.
#include "sl_device.h"
#include "sl_internal.h"

namespace {

constexpr int CAND_CAP = 512;       // LDS candidate list, entries
constexpr int CAND_SLOTS = CAND_CAP / 64;

struct SelectArgs {
    const SlChunkDesc *desc;
    const int *chunk_tensor;
    const SlTensorDev *tensors;
    float *e;
    const float *delta;
    float beta;
    int frozen;
    int k;
    float *vals;            // [n_chunks * k] selected values, canonical order
    double *leafA;          // [2][n_chunks] per-chunk tree sums of x and x*x
    unsigned char *payload;
    long long n_chunks;
};

SL_DEV int key_of(float x) { return (int)(__float_as_uint(x) & 0x7FFFFFFFu); }

// Largest T in [lo, hi] with count_ge(T) >= k, given count_ge(lo) >= k and
// 0 <= lo <= hi.  All values are wave-uniform.
template <class CountGE>
SL_DEV int bisect_kth(int lo, int hi, int k, CountGE count_ge)
{
    if (lo >= hi) return lo;
    const int top = 31 - __clz(lo ^ hi);
    int T = hi & ~(int)((2u << top) - 1u);
    for (int b = top; b >= 0; --b) {
        const int cand = T | (1 << b);
        if (count_ge(cand) >= k) T = cand;
    }
    return T;
}

template <int GPL>
SL_DEV void select_chunk(const SelectArgs &A, unsigned char *smem)
{
    const int lane = threadIdx.x;
    const long long c = blockIdx.x;
    const SlChunkDesc d = A.desc[c];
    const int k = A.k;

    int key[64];
    unsigned sg0 = 0, sg1 = 0;   // sign of register r at bit 31 - (r & 31) of sg[r / 32]

    // ---------------------------------------------------------------- a = beta*e + delta
    {
        float *ec = A.e + d.base;
        const float *dc = A.delta + d.base;
        const int lr = lane >> 4, lc = (lane & 15) * 4;
        const unsigned stride = (unsigned)d.stride;
        if (d.flags & SLC_FULL) {
            float4 ev[16], dv[16];
            const unsigned o0 = lr * stride + lc;
            if (!A.frozen) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    ev[i] = *reinterpret_cast<const float4 *>(ec + (o0 + 4u * i * stride));
            }
#pragma unroll
            for (int i = 0; i < 16; ++i)
                dv[i] = *reinterpret_cast<const float4 *>(dc + (o0 + 4u * i * stride));
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float4 a;
                if (!A.frozen) {
                    a.x = fmaf(A.beta, ev[i].x, dv[i].x);
                    a.y = fmaf(A.beta, ev[i].y, dv[i].y);
                    a.z = fmaf(A.beta, ev[i].z, dv[i].z);
                    a.w = fmaf(A.beta, ev[i].w, dv[i].w);
                    *reinterpret_cast<float4 *>(ec + (o0 + 4u * i * stride)) = a;
                } else {
                    a = dv[i];
                }
                const float av[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    const int r = 4 * i + cc;
                    const unsigned u = __float_as_uint(av[cc]);
                    key[r] = (int)(u & 0x7FFFFFFFu);
                    if (r < 32) sg0 = (sg0 << 1) | (u >> 31);
                    else sg1 = (sg1 << 1) | (u >> 31);
                }
            }
        } else {
            const int rows = d.rows, cols = d.cols, last_cols = d.last_cols;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = 4 * i + lr;
                const int lim = row < rows - 1 ? cols : (row == rows - 1 ? last_cols : 0);
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    const int r = 4 * i + cc;
                    const int col = lc + cc;
                    unsigned u = 0;
                    int kk = -1;
                    if (col < lim) {
                        const unsigned o = row * stride + col;
                        float a;
                        if (!A.frozen) {
                            a = fmaf(A.beta, ec[o], dc[o]);
                            ec[o] = a;
                        } else {
                            a = dc[o];
                        }
                        u = __float_as_uint(a);
                        kk = (int)(u & 0x7FFFFFFFu);
                    }
                    key[r] = kk;
                    if (r < 32) sg0 = (sg0 << 1) | (u >> 31);
                    else sg1 = (sg1 << 1) | (u >> 31);
                }
            }
        }
    }

    auto count_regs = [&](int x) {
        int n = 0;
#pragma unroll
        for (int r = 0; r < 64; ++r) n += sl_popc(sl_ballot(key[r] >= x));
        return n;
    };

    // ---------------------------------------------------------------- threshold T
    int T, n_ge;
    int *cand = reinterpret_cast<int *>(smem);
    if constexpr (GPL > 0) {
        constexpr int G = GPL;
        // group g of a lane = its registers r with r % G == g (interleaved, so
        // that partial chunks spread their valid positions over all groups)
        int gm[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            int m = key[g];
#pragma unroll
            for (int r = g + G; r < 64; r += G) m = max(m, key[r]);
            gm[g] = m;
        }
        int lmin = gm[0], lmax = gm[0];
#pragma unroll
        for (int g = 1; g < G; ++g) lmin = min(lmin, gm[g]), lmax = max(lmax, gm[g]);
        const int hi = sl_wave_max(lmax);               // largest key of the chunk (>= 0)
        const int lo = max(sl_wave_min(lmin), 0);
        // L = k-th largest group maximum: a lower bound of T, because k distinct
        // elements are >= L.  With fewer than k non-empty groups there is no
        // such bound and L = 0 keeps every valid key.
        auto count_gm = [&](int x) {
            int n = 0;
#pragma unroll
            for (int g = 0; g < G; ++g) n += sl_popc(sl_ballot(gm[g] >= x));
            return n;
        };
        const int L = count_gm(lo) >= k ? bisect_kth(lo, hi, k, count_gm) : 0;
        // compact the keys >= L into LDS (order irrelevant here)
        int ncand = 0;
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            const bool f = key[r] >= L;
            const unsigned long long m = sl_ballot(f);
            const int pos = ncand + sl_mbcnt(m);
            if (f && pos < CAND_CAP) cand[pos] = key[r];
            ncand += sl_popc(m);
        }
        __syncthreads();
        if (ncand <= CAND_CAP) {
            int cr[CAND_SLOTS];
            const int nslots = (ncand + 63) >> 6;
#pragma unroll
            for (int s = 0; s < CAND_SLOTS; ++s) {
                const int p = s * 64 + lane;
                cr[s] = (s < nslots && p < ncand) ? cand[p] : -1;
            }
            auto count_cand = [&](int x) {
                int n = 0;
#pragma unroll
                for (int s = 0; s < CAND_SLOTS; ++s)
                    if (s < nslots) n += sl_popc(sl_ballot(cr[s] >= x));
                return n;
            };
            T = bisect_kth(L, hi, k, count_cand);
            n_ge = count_cand(T);
        } else {
            T = bisect_kth(L, hi, k, count_regs);
            n_ge = count_regs(T);
        }
        __syncthreads();
    } else {
        int lmax = key[0];
#pragma unroll
        for (int r = 1; r < 64; ++r) lmax = max(lmax, key[r]);
        const int hi = sl_wave_max(lmax);
        T = bisect_kth(0, hi, k, count_regs);
        n_ge = count_regs(T);
    }

    // ---------------------------------------------------------------- ordered compaction
    float *sel_val = reinterpret_cast<float *>(smem);
    unsigned short *sel_idx = reinterpret_cast<unsigned short *>(smem + 4 * (size_t)k);
    const bool ties = n_ge != k;            // more keys equal to T than slots left
    // need = k - #(key > T): number of tie entries to take, lowest indices first
    int need = 0;
    if (ties) {
        int n_gt = 0;
#pragma unroll
        for (int r = 0; r < 64; ++r) n_gt += sl_popc(sl_ballot(key[r] > T));
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
                    sel_val[pos] = __uint_as_float((unsigned)key[r] | sign);
                    sel_idx[pos] = (unsigned short)(256 * i + 4 * lane + cc);
                    ++pos;
                }
            }
        }
        base += cnt;
    }
    __syncthreads();

    // ---------------------------------------------------------------- outputs
    const int t = A.chunk_tensor[c];
    const SlTensorDev td = A.tensors[t];
    const long long rec_bytes = (long long)7 * k / 4;
    unsigned char *rec = A.payload + td.pay_off + 16 + (c - td.chunk0) * rec_bytes;

    for (int p = lane; p < k; p += 64) A.vals[c * k + p] = sel_val[p];

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

    // per-chunk leaves of the quantizer's mean / variance sums
    double *scratch = reinterpret_cast<double *>(smem + 6 * (size_t)k + 8 - ((6 * (size_t)k) & 7));
    const double s1 = sl_chunk_tree(k, lane, scratch, [&](int s) {
        const int p = s * 64 + lane;
        return p < k ? (double)sel_val[p] : 0.0;
    });
    const double s2 = sl_chunk_tree(k, lane, scratch, [&](int s) {
        const int p = s * 64 + lane;
        const double x = p < k ? (double)sel_val[p] : 0.0;
        return x * x;
    });
    if (lane == 0) {
        A.leafA[c] = s1;
        A.leafA[A.n_chunks + c] = s2;
    }
}

template <int GPL>
__global__ void __launch_bounds__(64) k_select(SelectArgs A)
{
    extern __shared__ __align__(16) unsigned char smem[];
    select_chunk<GPL>(A, smem);
}

}  // namespace

static size_t select_lds_bytes(int k)
{
    size_t sel = 6 * (size_t)k;
    sel = (sel + 15) / 8 * 8;          // room for the 8-byte alignment of the tree scratch
    size_t need = sel + 64 * sizeof(double);
    size_t cand = CAND_CAP * sizeof(int);
    return need > cand ? need : cand;
}

int slk_select(const sl_plan *p, float *e, const float *delta, float beta, int frozen,
               unsigned char *payload, unsigned char *ws, hipStream_t st)
{
    if (p->n_chunks == 0) return SL_OK;
    SelectArgs A;
    A.desc = p->d_desc;
    A.chunk_tensor = p->d_chunk_tensor;
    A.tensors = p->d_tensors;
    A.e = e;
    A.delta = delta;
    A.beta = beta;
    A.frozen = frozen;
    A.k = p->k;
    A.vals = reinterpret_cast<float *>(ws + p->ws_vals);
    A.leafA = reinterpret_cast<double *>(ws + p->ws_leafA);
    A.payload = payload;
    A.n_chunks = p->n_chunks;
    const dim3 grid((unsigned)p->n_chunks), block(64);
    const size_t lds = select_lds_bytes(p->k);
    const int k = p->k;
    if (k <= 32) hipLaunchKernelGGL(k_select<1>, grid, block, lds, st, A);
    else if (k <= 64) hipLaunchKernelGGL(k_select<2>, grid, block, lds, st, A);
    else if (k <= 128) hipLaunchKernelGGL(k_select<4>, grid, block, lds, st, A);
    else if (k <= 256) hipLaunchKernelGGL(k_select<8>, grid, block, lds, st, A);
    else hipLaunchKernelGGL(k_select<0>, grid, block, lds, st, A);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    return SL_OK;
}
