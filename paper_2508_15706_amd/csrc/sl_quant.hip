// Kernels B-E of sl_compress: the per-tensor 2-bit statistical quantizer
// (Section 4, experimental set-up) and the error-feedback residual (Eq. (2)
// line 2, Algorithm 1 error update).
//
//   B  per tensor: fixed-tree fp64 sums of x and x*x over its selected values
//      -> mean mu and T = 9*var (squared distance of the outer bin edges);
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
        tstat[blockIdx.x].T = 9.0 * var;
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
    int lds_per_wave;
};

// One wave per chunk, several independent waves per workgroup.
__global__ void __launch_bounds__(256) k_codes(CodeArgs A)
{
    extern __shared__ __align__(16) unsigned char smem_all[];
    const int lane = threadIdx.x & 63, k = A.k;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= A.n_chunks) return;
    unsigned char *smem = smem_all + (size_t)wave * A.lds_per_wave;
    const SlChunkDesc d = A.desc[c];
    const double mu = A.tstat[d.tensor].mu, T = A.tstat[d.tensor].T;
    unsigned char *code_lds = smem;                                   // k bytes
    double *scratch = reinterpret_cast<double *>(smem + ((k + 7) & ~7));
    const float *x = A.vals + c * k;

    int n_b[4] = {0, 0, 0, 0};
    for (int s = 0; s * 64 < k; ++s) {
        const int p = s * 64 + lane;
        int code = -1;
        if (p < k) {
            const double d = (double)x[p] - mu;
            const double dd = d * d;
            code = d < 0.0 ? (dd > T ? 0 : 1) : (dd >= T ? 3 : 2);
            code_lds[p] = (unsigned char)code;
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) n_b[b] += sl_popc(sl_ballot(code == b));
    }
    sl_wave_sync();

    // codes, four per byte, entry m in bits 2*(m mod 4)
    unsigned char *rec = A.payload + d.rec_off + 3 * k / 2;
    if ((k & 15) == 0) {
        unsigned *rw = reinterpret_cast<unsigned *>(rec);
        for (int w = lane; w < k / 16; w += 64) {
            unsigned word = 0;
#pragma unroll
            for (int q = 0; q < 16; ++q) word |= (unsigned)code_lds[16 * w + q] << (2 * q);
            rw[w] = word;
        }
    } else {
        for (int b = lane; b < k / 4; b += 64) {
            unsigned v = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) v |= (unsigned)code_lds[4 * b + q] << (2 * q);
            rec[b] = (unsigned char)v;
        }
    }

#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const double sb = sl_chunk_tree(k, lane, scratch, [&](int s) {
            const int p = s * 64 + lane;
            return (p < k && code_lds[p] == b) ? (double)x[p] : 0.0;
        });
        if (lane == 0) {
            A.leafC[b * A.n_chunks + c] = sb;
            A.cnt[b * A.n_chunks + c] = (unsigned)n_b[b];
        }
    }
}

// ------------------------------------------------------------------ kernel D
__global__ void __launch_bounds__(RED_THREADS)
k_tensor_lut(const SlTensorDev *tensors, const double *leafC, const unsigned *cnt,
             long long n_chunks_total, int k, SlTensorStat *tstat, unsigned char *payload)
{
    __shared__ RedShared sh;
    const SlTensorDev td = tensors[blockIdx.x];
    const int tid = threadIdx.x;
    if (tid < 4) sh.cnt[tid] = 0ull;
    __syncthreads();
    for (int b = 0; b < 4; ++b) {
        unsigned long long part = 0;
        for (long long i = tid; i < td.n_chunks; i += RED_THREADS)
            part += cnt[b * n_chunks_total + td.chunk0 + i];
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) part += __shfl_xor(part, s);
        if ((tid & 63) == 0 && part) atomicAdd(&sh.cnt[b], part);   // integer: order-free
    }
    __syncthreads();
    float lut[4];
    for (int b = 0; b < 4; ++b) {
        const double Sb = block_tree_sum(leafC + b * n_chunks_total + td.chunk0, td.n_chunks, sh);
        const unsigned long long nb = sh.cnt[b];
        float cen = nb ? (float)(Sb / (double)nb) : 0.0f;
        if (cen == 0.0f) cen = 0.0f;        // never -0.0f on the wire
        lut[b] = cen;
    }
    if (tid == 0) {
#pragma unroll
        for (int b = 0; b < 4; ++b) tstat[blockIdx.x].lut[b] = lut[b];
        *reinterpret_cast<float4 *>(payload + td.pay_off) = make_float4(lut[0], lut[1], lut[2], lut[3]);
    }
    // zero the padding that rounds the tensor block up to 16 bytes
    const long long used = 16 + td.n_chunks * ((long long)7 * k / 4);
    if (tid < td.block_bytes - used) payload[td.pay_off + used + tid] = 0;
}

// ------------------------------------------------------------------ kernel E
struct ResidualArgs {
    const SlChunkDesc *desc;
    const float *vals;              // the selected values a, or null: read them from e
    const unsigned char *payload;
    float *e;
    long long n_chunks;
    int k;
};

__global__ void __launch_bounds__(256) k_residual(ResidualArgs A)
{
    const int lane = threadIdx.x & 63, k = A.k;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= A.n_chunks) return;
    const SlChunkDesc d = A.desc[c];
    const float4 lut = *reinterpret_cast<const float4 *>(A.payload + sl_lut_off(d, k));
    const unsigned char *rec = A.payload + d.rec_off;
    const unsigned char *codes = rec + 3 * k / 2;
    float *ec = A.e + d.base;
    for (int m = lane; m < k; m += 64) {
        const int b = (3 * m) >> 1;
        const unsigned w = (unsigned)rec[b] | ((unsigned)rec[b + 1] << 8);
        const unsigned j = (m & 1) ? (w >> 4) : (w & 0xFFFu);
        const unsigned code = (codes[m >> 2] >> (2 * (m & 3))) & 3u;
        const float q = code == 0 ? lut.x : code == 1 ? lut.y : code == 2 ? lut.z : lut.w;
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

int slk_quantize(const sl_plan *p, float *e, int skip_residual, unsigned char *payload,
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
    C.lds_per_wave = ((k + 15) & ~15) + 64 * (int)sizeof(double);
    const int wpb = 4;
    const unsigned nblk = (unsigned)((p->n_chunks + wpb - 1) / wpb);
    hipLaunchKernelGGL(k_codes, dim3(nblk), dim3(64 * wpb), (size_t)C.lds_per_wave * wpb, st, C);
    if ((rc = check_launch())) return rc;
    sl_prof_mark(p, SL_PROF_CODES, st);

    hipLaunchKernelGGL(k_tensor_lut, dim3(p->n_tensors), dim3(RED_THREADS), 0, st, p->d_tensors,
                       leafC, cnt, (long long)p->n_chunks, k, tstat, payload);
    if ((rc = check_launch())) return rc;
    sl_prof_mark(p, SL_PROF_LUT, st);

    if (!skip_residual) {
        if ((rc = launch_residual(p, e, vals, payload, st))) return rc;
        sl_prof_mark(p, SL_PROF_RESIDUAL, st);
    }
    return SL_OK;
}
