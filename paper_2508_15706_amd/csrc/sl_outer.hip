// Dense outer steps of the DiLoCo family (Eq. (1): DiLoCo's Nesterov outer
// momentum; Section 3.2: DiLoCo-LOM; appendix "Exact algorithmic description of
// DiLoCo variants").  They are the dense counterparts of the sparse aggregate
// in sl_apply.hip and walk the same chunk work list, so that elements of the
// arenas that belong to no tensor are never touched.
//
//   k_lom_direction   m <- mu*m + delta ; dir <- delta + mu*m         (one worker)
//   k_dense_avg_apply avg = (1/R) sum_r dirs[r], r ascending from +0.0f;
//                     [m <- mu*m + avg ; avg <- avg + mu*m] ; theta <- theta - lr*avg
//
// Every "c*y + z" is one fp32 fused multiply-add.  Both kernels are pure
// streams: one wavefront owns one chunk and moves it in two halves of eight
// 16-byte accesses per lane per stream, so that many workgroups stay resident.
#include "sl_device.h"
#include "sl_internal.h"

// 16-byte accesses per lane and stream that are in flight together (half a chunk; a quarter
// and a whole chunk measured the same within the run-to-run spread of these kernels)
#ifndef SL_LOM_STEP
#define SL_LOM_STEP 8
#endif
#ifndef SL_DENSE_STEP
#define SL_DENSE_STEP 8
#endif
namespace {

struct LomArgs {
    const SlChunkDesc *desc;
    float *m;
    const float *delta;
    float *dir;
    float mu;
    long long n_chunks;
};

__global__ void __launch_bounds__(256) k_lom_direction(LomArgs A)
{
    const int lane = threadIdx.x & 63;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= A.n_chunks) return;
    const SlChunkDesc d = A.desc[c];
    float *mc = A.m + d.base;
    const float *dc = A.delta + d.base;
    float *oc = A.dir + d.base;
    const int lr = lane >> 4, lc = (lane & 15) * 4;
    const unsigned stride = (unsigned)d.stride;
    if (d.flags & SLC_FULL) {
        const unsigned o0 = 4u * (lr * stride + lc), step = 16u * stride;
        constexpr int S = SL_LOM_STEP;
#pragma unroll
        for (int q = 0; q < 16 / S; ++q) {
            sl_f4 mv[S], dv[S];
#pragma unroll
            for (int u = 0; u < S; ++u) mv[u] = sl_load_stream_at(mc, (S * q + u) * step, o0);
#pragma unroll
            for (int u = 0; u < S; ++u) dv[u] = sl_load_stream_at(dc, (S * q + u) * step, o0);
#pragma unroll
            for (int u = 0; u < S; ++u) {
                sl_f4 m = mv[u], g = dv[u], o;
                m.x = fmaf(A.mu, m.x, g.x), m.y = fmaf(A.mu, m.y, g.y);
                m.z = fmaf(A.mu, m.z, g.z), m.w = fmaf(A.mu, m.w, g.w);
                o.x = fmaf(A.mu, m.x, g.x), o.y = fmaf(A.mu, m.y, g.y);
                o.z = fmaf(A.mu, m.z, g.z), o.w = fmaf(A.mu, m.w, g.w);
                sl_store_stream_at(mc, (S * q + u) * step, o0, m);
                sl_store_stream_at(oc, (S * q + u) * step, o0, o);
            }
        }
    } else {
        const int rows = d.rows, cols = d.cols, last_cols = d.last_cols;
        for (int i = 0; i < 16; ++i) {
            const int row = 4 * i + lr;
            const int lim = row < rows - 1 ? cols : (row == rows - 1 ? last_cols : 0);
            for (int cc = 0; cc < 4; ++cc) {
                const int col = lc + cc;
                if (col < lim) {
                    const unsigned o = row * stride + col;
                    const float g = dc[o];
                    const float m = fmaf(A.mu, mc[o], g);
                    mc[o] = m;
                    oc[o] = fmaf(A.mu, m, g);
                }
            }
        }
    }
}

struct DenseArgs {
    const SlChunkDesc *desc;
    float *theta;
    float *mom;              // global momentum (Eq. (1)), or null
    float neg_lr, inv_R, mu;
    int R;
    long long n_chunks;
    const float *dirs[SL_MAX_WORKERS];
};

template <bool NESTEROV>
__global__ void __launch_bounds__(256) k_dense_avg_apply(DenseArgs A)
{
    const int lane = threadIdx.x & 63;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= A.n_chunks) return;
    const SlChunkDesc d = A.desc[c];
    float *tc = A.theta + d.base;
    float *mc = NESTEROV ? A.mom + d.base : nullptr;
    const int lr = lane >> 4, lc = (lane & 15) * 4;
    const unsigned stride = (unsigned)d.stride;
    const int R = A.R;
    if (d.flags & SLC_FULL) {
        const unsigned o0 = 4u * (lr * stride + lc), step = 16u * stride;
        constexpr int S = SL_DENSE_STEP;
#pragma unroll 1
        for (int q = 0; q < 16 / S; ++q) {
            sl_f4 th[S], mo[NESTEROV ? S : 1], acc[S];
#pragma unroll
            for (int u = 0; u < S; ++u) th[u] = sl_load_stream_at(tc, (S * q + u) * step, o0);
            if constexpr (NESTEROV) {
#pragma unroll
                for (int u = 0; u < S; ++u) mo[u] = sl_load_stream_at(mc, (S * q + u) * step, o0);
            }
#pragma unroll
            for (int u = 0; u < S; ++u) acc[u] = sl_f4{0.f, 0.f, 0.f, 0.f};
            for (int r = 0; r < R; ++r) {                   // r ascending: the order is part of the result
                const float *gc = A.dirs[r] + d.base;
                sl_f4 g[S];
#pragma unroll
                for (int u = 0; u < S; ++u) g[u] = sl_load_stream_at(gc, (S * q + u) * step, o0);
#pragma unroll
                for (int u = 0; u < S; ++u) acc[u] = acc[u] + g[u];
            }
#pragma unroll
            for (int u = 0; u < S; ++u) {
                sl_f4 g = acc[u] * A.inv_R;
                if constexpr (NESTEROV) {
                    sl_f4 m = mo[u];
                    m.x = fmaf(A.mu, m.x, g.x), m.y = fmaf(A.mu, m.y, g.y);
                    m.z = fmaf(A.mu, m.z, g.z), m.w = fmaf(A.mu, m.w, g.w);
                    sl_store_stream_at(mc, (S * q + u) * step, o0, m);
                    g.x = fmaf(A.mu, m.x, g.x), g.y = fmaf(A.mu, m.y, g.y);
                    g.z = fmaf(A.mu, m.z, g.z), g.w = fmaf(A.mu, m.w, g.w);
                }
                sl_f4 v = th[u];
                v.x = fmaf(A.neg_lr, g.x, v.x), v.y = fmaf(A.neg_lr, g.y, v.y);
                v.z = fmaf(A.neg_lr, g.z, v.z), v.w = fmaf(A.neg_lr, g.w, v.w);
                sl_store_stream_at(tc, (S * q + u) * step, o0, v);
            }
        }
    } else {
        const int rows = d.rows, cols = d.cols, last_cols = d.last_cols;
        for (int i = 0; i < 16; ++i) {
            const int row = 4 * i + lr;
            const int lim = row < rows - 1 ? cols : (row == rows - 1 ? last_cols : 0);
            for (int cc = 0; cc < 4; ++cc) {
                const int col = lc + cc;
                if (col < lim) {
                    const unsigned o = row * stride + col;
                    float acc = 0.0f;
                    for (int r = 0; r < R; ++r) acc = acc + (A.dirs[r] + d.base)[o];
                    float g = acc * A.inv_R;
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

int check_launch()
{
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    return SL_OK;
}

}  // namespace

int slk_lom_direction(const sl_plan *p, float *m, const float *delta, float mu, float *dir, hipStream_t st)
{
    if (p->n_chunks == 0) return SL_OK;
    LomArgs A;
    A.desc = p->d_desc;
    A.m = m;
    A.delta = delta;
    A.dir = dir;
    A.mu = mu;
    A.n_chunks = p->n_chunks;
    hipLaunchKernelGGL(k_lom_direction, dim3((unsigned)((p->n_chunks + 3) / 4)), dim3(256), 0, st, A);
    return check_launch();
}

int slk_dense_avg_apply(const sl_plan *p, float *theta, float *mom, const float *const *dirs, int R, float lr,
                        float mu, hipStream_t st)
{
    if (p->n_chunks == 0) return SL_OK;
    DenseArgs A;
    A.desc = p->d_desc;
    A.theta = theta;
    A.mom = mom;
    A.neg_lr = -lr;
    A.inv_R = 1.0f / (float)R;
    A.mu = mu;
    A.R = R;
    A.n_chunks = p->n_chunks;
    for (int r = 0; r < SL_MAX_WORKERS; ++r) A.dirs[r] = r < R ? dirs[r] : nullptr;
    const dim3 grid((unsigned)((p->n_chunks + 3) / 4)), block(256);
    if (mom) hipLaunchKernelGGL(k_dense_avg_apply<true>, grid, block, 0, st, A);
    else hipLaunchKernelGGL(k_dense_avg_apply<false>, grid, block, 0, st, A);
    return check_launch();
}
