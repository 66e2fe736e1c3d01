// Host side of the C ABI: plan construction (chunk work list), argument
// validation and kernel sequencing.  See include/sparseloco.h for the contract.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "sl_internal.h"

static thread_local char g_hip_error[256] = "";

void sl_note_hip_error(hipError_t e)
{
    std::strncpy(g_hip_error, hipGetErrorString(e), sizeof(g_hip_error) - 1);
    g_hip_error[sizeof(g_hip_error) - 1] = 0;
}

static int hip_fail(hipError_t e)
{
    sl_note_hip_error(e);
    return SL_ERR_HIP;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// limits of a plan (documented at sl_plan_create)
static const int64_t SL_MAX_TENSOR_ELEMS = (int64_t)1 << 46;
static const int64_t SL_MAX_CHUNKS = (int64_t)1 << 27;

extern "C" int sl_profile_end(sl_plan *p, double *ms, int *calls);

extern "C" {

const char *sl_strerror(int status)
{
    switch (status) {
        case SL_OK: return "ok";
        case SL_ERR_INVALID_ARG: return "invalid argument";
        case SL_ERR_BAD_PAYLOAD: return "malformed payload";
        case SL_ERR_HIP: return "HIP runtime error";
        case SL_ERR_NOMEM: return "out of memory";
        case SL_ERR_DEVICE: return "plan belongs to another device";
        case SL_ERR_TOO_LARGE: return "plan needs more scratch memory than the entry point without allocations holds";
        default: return "unknown status";
    }
}

const char *sl_last_hip_error(void) { return g_hip_error; }

int sl_plan_create(const sl_tensor *tensors, int n_tensors, int k, sl_plan **out)
{
    return sl_plan_create_bits(tensors, n_tensors, k, 2, out);
}

int sl_plan_value_bits(const sl_plan *p) { return p ? p->bits : -1; }

int sl_plan_create_bits(const sl_tensor *tensors, int n_tensors, int k, int value_bits, sl_plan **out)
{
    if (!out) return SL_ERR_INVALID_ARG;
    *out = nullptr;
    if (n_tensors < 0 || (n_tensors > 0 && !tensors)) return SL_ERR_INVALID_ARG;
    if (k < 4 || k > SL_CHUNK || (k & 3)) return SL_ERR_INVALID_ARG;
    const int bits = value_bits;
    if (!(bits == 1 || bits == 2 || bits == 3 || bits == 4 || bits == 32)) return SL_ERR_INVALID_ARG;
    if (bits != 2 && (k & 7)) return SL_ERR_INVALID_ARG;   // records must end on a byte

    const int64_t rec = sl_rec_bytes(k, bits), hdr = sl_hdr_bytes(bits);
    const int nbins = bits == 32 ? 0 : 1 << bits;
    std::vector<SlChunkDesc> desc;
    std::vector<SlTensorDev> tdev;
    std::vector<SlGroup> groups;
    int64_t n_elements = 0, n_partial = 0;
    size_t pay = 0;

    // tensors must not overlap: results would depend on processing order
    try {
        tdev.resize((size_t)n_tensors);
        std::vector<std::pair<int64_t, int64_t>> span;
        span.reserve((size_t)n_tensors);
        int64_t total_chunks = 0;
        for (int t = 0; t < n_tensors; ++t) {
            const sl_tensor &T = tensors[t];
            if (T.rows < 1 || T.cols < 1 || T.offset < 0 || (T.offset & 3) || T.reserved != 0)
                return SL_ERR_INVALID_ARG;
            if (T.layout != SL_LAYOUT_FLAT && T.layout != SL_LAYOUT_TILE64) return SL_ERR_INVALID_ARG;
            if (T.rows > SL_MAX_TENSOR_ELEMS / T.cols) return SL_ERR_INVALID_ARG;   // no overflow in the product
            if (T.offset > ((int64_t)1 << 60)) return SL_ERR_INVALID_ARG;
            if (T.layout == SL_LAYOUT_TILE64 && T.cols > (int64_t)1 << 23) return SL_ERR_INVALID_ARG;
            span.emplace_back(T.offset, T.offset + T.rows * T.cols);
            // the work list is built only once its length is known to be within the limit
            total_chunks += T.layout == SL_LAYOUT_TILE64 ? ((T.rows + 63) / 64) * ((T.cols + 63) / 64)
                                                         : (T.rows * T.cols + SL_CHUNK - 1) / SL_CHUNK;
            if (total_chunks > SL_MAX_CHUNKS) return SL_ERR_INVALID_ARG;
        }
        std::sort(span.begin(), span.end());
        for (size_t i = 1; i < span.size(); ++i)
            if (span[i].first < span[i - 1].second) return SL_ERR_INVALID_ARG;
    } catch (const std::bad_alloc &) {
        return SL_ERR_NOMEM;
    }

    try {
        for (int t = 0; t < n_tensors; ++t) {
            const sl_tensor &T = tensors[t];
            SlTensorDev &D = tdev[(size_t)t];
            D.chunk0 = (long long)desc.size();
            if (T.layout == SL_LAYOUT_TILE64) {
                const int64_t tr = (T.rows + 63) / 64, tc = (T.cols + 63) / 64;
                for (int64_t a = 0; a < tr; ++a)
                    for (int64_t b = 0; b < tc; ++b) {
                        SlChunkDesc d;
                        d.base = T.offset + a * 64 * T.cols + b * 64;
                        d.stride = (int)T.cols;
                        const int64_t rv = std::min<int64_t>(64, T.rows - a * 64);
                        const int64_t cv = std::min<int64_t>(64, T.cols - b * 64);
                        if (rv * cv < k) return SL_ERR_INVALID_ARG;
                        d.rows = (unsigned char)rv;
                        d.cols = d.last_cols = (unsigned char)cv;
                        d.flags = (rv == 64 && cv == 64) ? SLC_FULL : 0;
                        d.tensor = t;
                        d.local_chunk = (int)(a * tc + b);
                        d.rec_off = (long long)pay + hdr + (long long)d.local_chunk * rec;
                        desc.push_back(d);
                    }
            } else {
                const int64_t n = T.rows * T.cols;
                for (int64_t a = 0; a * SL_CHUNK < n; ++a) {
                    SlChunkDesc d;
                    d.base = T.offset + a * SL_CHUNK;
                    d.stride = 64;
                    const int64_t nv = std::min<int64_t>(SL_CHUNK, n - a * SL_CHUNK);
                    if (nv < k) return SL_ERR_INVALID_ARG;
                    d.rows = (unsigned char)((nv + 63) / 64);
                    d.cols = 64;
                    d.last_cols = (unsigned char)(nv - (int64_t)(d.rows - 1) * 64);
                    d.flags = nv == SL_CHUNK ? SLC_FULL : 0;
                    d.tensor = t;
                    d.local_chunk = (int)a;
                    d.rec_off = (long long)pay + hdr + (long long)d.local_chunk * rec;
                    desc.push_back(d);
                }
            }
            D.n_chunks = (long long)desc.size() - D.chunk0;
            D.pay_off = (long long)pay;
            D.block_bytes = (long long)align_up((size_t)(hdr + D.n_chunks * rec), 16);
            D.group0 = (long long)groups.size();
            for (long long g = 0; g * SL_RICE_GROUP < D.n_chunks; ++g) groups.push_back(SlGroup{t, (int)g});
            pay += (size_t)D.block_bytes;
            n_elements += T.rows * T.cols;
        }
    } catch (const std::bad_alloc &) {
        return SL_ERR_NOMEM;
    }
    for (const SlChunkDesc &d : desc) n_partial += !(d.flags & SLC_FULL);

    sl_plan *p = new (std::nothrow) sl_plan();
    if (!p) return SL_ERR_NOMEM;
    std::memset(p, 0, sizeof(*p));
    p->k = k;
    p->bits = bits;
    p->rec_bytes = (int)rec;
    p->hdr_bytes = (int)hdr;
    p->n_tensors = n_tensors;
    p->n_chunks = (int64_t)desc.size();
    p->n_elements = n_elements;
    p->n_partial = n_partial;
    p->payload_bytes = pay;

    size_t off = 0;
    p->ws_vals = off;   off = align_up(off + (size_t)p->n_chunks * k * sizeof(float), 256);
    p->ws_leafA = off;  off = align_up(off + (size_t)p->n_chunks * 2 * sizeof(double), 256);
    p->ws_leafC = off;  off = align_up(off + (size_t)p->n_chunks * nbins * sizeof(double), 256);
    p->ws_cnt = off;    off = align_up(off + (size_t)p->n_chunks * nbins * sizeof(unsigned), 256);
    p->ws_tstat = off;  off = align_up(off + (size_t)n_tensors * sizeof(SlTensorStat), 256);
    p->ws_bytes = off ? off : 256;
    p->n_groups = (int64_t)groups.size();
    p->codes_wave_below = 32768;
    {
        // the coded format's sizes, its upper bound and the scratch its writers need
        SlCodedGeom &g = p->cg;
        g.k = k, g.bits = bits;
        g.b = sl_rice_param(k);
        g.qmax = (SL_CHUNK - k) >> g.b;
        g.qf = g.qmax < 256 ? 1 : 2;
        g.dent = 4 + SL_RICE_GROUP * g.qf;
        g.rem_bytes = (k * g.b + 31) / 32 * 4;
        g.val_bytes = k * bits / 8;
        g.cfix = (g.rem_bytes + g.val_bytes + 3) / 4 * 4;
        g.hdr = (int)hdr;
        g.ua = (k + g.qmax + 31) / 32;
        size_t pos = 16, words = 0;
        for (int t = 0; t < n_tensors; ++t) {
            SlTensorDev &D = tdev[(size_t)t];
            const size_t ng = (size_t)((D.n_chunks + SL_RICE_GROUP - 1) / SL_RICE_GROUP);
            D.cblk_off = (long long)pos;
            D.cdir_off = D.cblk_off + hdr;
            D.cfix_off = D.cdir_off + (long long)(ng * (size_t)g.dent);
            D.cblk_bytes = (long long)align_up((size_t)hdr + ng * (size_t)g.dent + (size_t)D.n_chunks * (size_t)g.cfix, 16);
            pos += (size_t)D.cblk_bytes;
            for (long long c0 = 0; c0 < D.n_chunks; c0 += SL_RICE_GROUP)
                words += ((size_t)std::min<long long>(SL_RICE_GROUP, D.n_chunks - c0) * (size_t)(k + g.qmax) + 31) / 32;
        }
        g.section = (long long)pos;
        // run offsets travel as 32-bit word counts
        p->rice_max_bytes = words < ((size_t)1 << 32) ? align_up(pos + 4 * words, 16) : 0;
        p->ws_uvec = off;    off = align_up(off + (size_t)p->n_chunks * (size_t)g.ua * 4, 256);
        p->ws_qsum = off;    off = align_up(off + (size_t)p->n_chunks * 2, 256);
        p->ws_gwords = off;  off = align_up(off + groups.size() * 4, 256);
        p->ws_goff = off;    off = align_up(off + groups.size() * 4, 256);
        p->ws_twords = off;  off = align_up(off + ((size_t)n_tensors + 1) * 8, 256);
        p->ws_bytes = off;
    }

    hipError_t err = hipGetDevice(&p->device);
    if (err != hipSuccess) {
        delete p;
        return hip_fail(err);
    }
    {
        // the scratch array of sl_compress_noalloc: looked up now, with the plan's device current, so that
        // the entry point itself has nothing left to set up (a failure here is reported by that call)
        void *unused = nullptr;
        (void)sl_noalloc_scratch(p->device, &unused);
    }
    p->max_lds = 65536;
    {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, p->device) == hipSuccess &&
            v >= 32768)
            p->max_lds = v;
    }
    p->h_tensors = (SlTensorDev *)std::malloc(sizeof(SlTensorDev) * (size_t)std::max(1, n_tensors));
    if (!p->h_tensors) {
        delete p;
        return SL_ERR_NOMEM;
    }
    if (n_tensors) std::memcpy(p->h_tensors, tdev.data(), sizeof(SlTensorDev) * (size_t)n_tensors);

    if (p->n_chunks > 0) {
        const size_t b_desc = desc.size() * sizeof(SlChunkDesc),
                     b_t = (size_t)n_tensors * sizeof(SlTensorDev);
        std::vector<SlCodedDesc> cdesc;
        try {
            cdesc.resize(desc.size());
        } catch (const std::bad_alloc &) {
            sl_plan_destroy(p);
            return SL_ERR_NOMEM;
        }
        for (size_t i = 0; i < desc.size(); ++i) {
            const SlTensorDev &D = tdev[(size_t)desc[i].tensor];
            cdesc[i].lut_off = D.cblk_off;
            cdesc[i].dir_off = D.cdir_off + (long long)(desc[i].local_chunk / SL_RICE_GROUP) * p->cg.dent;
            cdesc[i].fix_off = D.cfix_off + (long long)desc[i].local_chunk * p->cg.cfix;
            cdesc[i].pos = desc[i].local_chunk % SL_RICE_GROUP;
            cdesc[i].reserved = 0;
        }
        if ((err = hipMalloc((void **)&p->d_desc, b_desc)) != hipSuccess ||
            (err = hipMalloc((void **)&p->d_cdesc, cdesc.size() * sizeof(SlCodedDesc))) != hipSuccess ||
            (err = hipMemcpy(p->d_cdesc, cdesc.data(), cdesc.size() * sizeof(SlCodedDesc),
                             hipMemcpyHostToDevice)) != hipSuccess ||
            (err = hipMalloc((void **)&p->d_tensors, b_t)) != hipSuccess ||
            (err = hipMalloc((void **)&p->d_groups, groups.size() * sizeof(SlGroup))) != hipSuccess ||
            (err = hipMemcpy(p->d_groups, groups.data(), groups.size() * sizeof(SlGroup),
                             hipMemcpyHostToDevice)) != hipSuccess ||
            (err = hipMemcpy(p->d_desc, desc.data(), b_desc, hipMemcpyHostToDevice)) != hipSuccess ||
            (err = hipMemcpy(p->d_tensors, tdev.data(), b_t, hipMemcpyHostToDevice)) != hipSuccess) {
            const int rc = err == hipErrorOutOfMemory ? SL_ERR_NOMEM : hip_fail(err);
            sl_plan_destroy(p);
            return rc;
        }
    }
    *out = p;
    return SL_OK;
}

int sl_plan_destroy(sl_plan *p)
{
    if (!p) return SL_OK;
    if (p->d_desc) (void)hipFree(p->d_desc);
    if (p->d_cdesc) (void)hipFree(p->d_cdesc);
    if (p->d_tensors) (void)hipFree(p->d_tensors);
    if (p->d_groups) (void)hipFree(p->d_groups);
    std::free(p->h_tensors);
    if (p->prof) {
        double ms[SL_PROF_PHASES];
        (void)sl_profile_end(p, ms, nullptr);
    }
    delete p;
    return SL_OK;
}

int64_t sl_plan_num_chunks(const sl_plan *p) { return p ? p->n_chunks : -1; }
int64_t sl_plan_num_elements(const sl_plan *p) { return p ? p->n_elements : -1; }
size_t sl_payload_bytes(const sl_plan *p) { return p ? p->payload_bytes : 0; }
size_t sl_workspace_bytes(const sl_plan *p) { return p ? p->ws_bytes : 0; }

size_t sl_payload_tensor_offset(const sl_plan *p, int t)
{
    if (!p || t < 0 || t >= p->n_tensors) return (size_t)-1;
    return (size_t)p->h_tensors[t].pay_off;
}

static int check_device(const sl_plan *p)
{
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return hip_fail(err);
    return dev == p->device ? SL_OK : SL_ERR_DEVICE;
}

static bool misaligned(const void *ptr, size_t a) { return ((uintptr_t)ptr & (a - 1)) != 0; }

}  // extern "C"

int sl_compress_impl(sl_plan *p, float *e, const float *delta, const float *theta_local, float beta,
                     int flags, const void *pending, void *payload, void *workspace, void *stream,
                     bool random, unsigned seed, void *coded, size_t coded_capacity)
{
    if (!p || !delta || !payload || !workspace) return SL_ERR_INVALID_ARG;
    if (coded && (p->rice_max_bytes == 0 || coded_capacity < p->rice_max_bytes || misaligned(coded, 16) ||
                  coded == payload || coded == pending || random))
        return SL_ERR_INVALID_ARG;
    if (flags & ~(SL_COMPRESS_EF_FROZEN | SL_COMPRESS_DEFER_RESIDUAL)) return SL_ERR_INVALID_ARG;
    const int frozen = (flags & SL_COMPRESS_EF_FROZEN) ? 1 : 0;
    const int defer = (flags & SL_COMPRESS_DEFER_RESIDUAL) ? 1 : 0;
    if (!frozen && !e) return SL_ERR_INVALID_ARG;
    if (frozen && (pending || defer)) return SL_ERR_INVALID_ARG;
    if (e == delta || (theta_local && (e == theta_local || delta == theta_local)) || pending == payload)
        return SL_ERR_INVALID_ARG;
    if (misaligned(e, 16) || misaligned(delta, 16) || misaligned(theta_local, 16) ||
        misaligned(payload, 16) || misaligned(pending, 16) || misaligned(workspace, 256))
        return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char *pay = static_cast<unsigned char *>(payload);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    sl_prof_mark(p, -1, st);
    if (random)
        rc = slk_select_random(p, e, delta, beta, frozen, static_cast<const unsigned char *>(pending), pay, ws,
                               seed, st);
    else
        rc = slk_select(p, e, delta, theta_local, beta, frozen, static_cast<const unsigned char *>(pending),
                        pay, static_cast<unsigned char *>(coded), ws, st);
    if (rc) return rc;
    sl_prof_mark(p, SL_PROF_SELECT, st);
    rc = slk_quantize(p, e, frozen || defer, pay, static_cast<unsigned char *>(coded), ws, st);
    if (rc || !coded) return rc;
    rc = slk_coded_finish(p, static_cast<unsigned char *>(coded), ws, st);
    sl_prof_mark(p, SL_PROF_INDEX, st);
    return rc;
}

extern "C" {

int sl_compress(sl_plan *p, float *e, const float *delta, float beta, int flags, const void *pending,
                void *payload, void *workspace, void *stream)
{
    return sl_compress_impl(p, e, delta, nullptr, beta, flags, pending, payload, workspace, stream);
}

int sl_compress_params(sl_plan *p, float *e, const float *theta_outer, const float *theta_local,
                       float beta, int flags, const void *pending, void *payload, void *workspace,
                       void *stream)
{
    if (!theta_local) return SL_ERR_INVALID_ARG;
    return sl_compress_impl(p, e, theta_outer, theta_local, beta, flags, pending, payload, workspace, stream);
}

int sl_compress_random_k(sl_plan *p, float *e, const float *delta, float beta, int flags, const void *pending,
                         void *payload, void *workspace, uint32_t seed, void *stream)
{
    return sl_compress_impl(p, e, delta, nullptr, beta, flags, pending, payload, workspace, stream, true, seed);
}

int sl_compress_coded(sl_plan *p, float *e, const float *delta, float beta, int flags, const void *pending,
                      void *record, void *coded, size_t coded_capacity, void *workspace, void *stream)
{
    if (!coded) return SL_ERR_INVALID_ARG;
    return sl_compress_impl(p, e, delta, nullptr, beta, flags, pending, record, workspace, stream, false, 0u,
                            coded, coded_capacity);
}

int sl_plan_set_codes_wave_below(sl_plan *p, int64_t n_chunks)
{
    if (!p || n_chunks < 0) return SL_ERR_INVALID_ARG;
    p->codes_wave_below = n_chunks;
    return SL_OK;
}

size_t sl_rice_max_bytes(const sl_plan *p) { return p ? p->rice_max_bytes : 0; }
size_t sl_coded_fixed_bytes(const sl_plan *p) { return p ? (size_t)p->cg.section : 0; }

int sl_rice_encode(sl_plan *p, const void *payload, void *out, size_t out_capacity, void *workspace,
                   void *stream)
{
    if (!p || !payload || !out || !workspace) return SL_ERR_INVALID_ARG;
    if (p->rice_max_bytes == 0 || out_capacity < p->rice_max_bytes || payload == out) return SL_ERR_INVALID_ARG;
    if (misaligned(payload, 16) || misaligned(out, 16) || misaligned(workspace, 256))
        return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    return slk_rice_encode(p, static_cast<const unsigned char *>(payload), static_cast<unsigned char *>(out),
                           static_cast<unsigned char *>(workspace), static_cast<hipStream_t>(stream));
}

int sl_rice_decode(sl_plan *p, const void *in, size_t in_bytes, void *payload, void *stream)
{
    if (!p || !in || !payload || in == payload) return SL_ERR_INVALID_ARG;
    if (p->rice_max_bytes == 0 || in_bytes < (size_t)p->cg.section) return SL_ERR_INVALID_ARG;
    if (misaligned(in, 16) || misaligned(payload, 16)) return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    const void *one[1] = {in};
    return slk_apply_coded(p, 2, nullptr, nullptr, 0.0f, static_cast<unsigned char *>(payload), one, &in_bytes, 1,
                           0.0f, static_cast<hipStream_t>(stream));
}

static int apply_coded(sl_plan *p, float *theta, float *momentum, float mu, const void *const *coded,
                       const size_t *coded_bytes, int R, float lr, void *stream)
{
    if (!p || !theta || !coded || !coded_bytes || R < 1 || R > SL_MAX_WORKERS) return SL_ERR_INVALID_ARG;
    if (p->rice_max_bytes == 0 || misaligned(theta, 16) || misaligned(momentum, 16)) return SL_ERR_INVALID_ARG;
    for (int r = 0; r < R; ++r)
        if (!coded[r] || misaligned(coded[r], 16) || coded_bytes[r] < (size_t)p->cg.section) return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    sl_prof_mark(p, -2, static_cast<hipStream_t>(stream));
    rc = slk_apply_coded(p, momentum ? 1 : 0, theta, momentum, mu, nullptr, coded, coded_bytes, R, lr,
                         static_cast<hipStream_t>(stream));
    sl_prof_mark(p, SL_PROF_APPLY, static_cast<hipStream_t>(stream));
    return rc;
}

int sl_decompress_avg_apply_coded(sl_plan *p, float *theta, const void *const *coded, const size_t *coded_bytes,
                                  int R, float lr, void *stream)
{
    return apply_coded(p, theta, nullptr, 0.0f, coded, coded_bytes, R, lr, stream);
}

int sl_decompress_avg_apply_nesterov_coded(sl_plan *p, float *theta, float *momentum, const void *const *coded,
                                           const size_t *coded_bytes, int R, float lr, float mu, void *stream)
{
    if (!momentum || momentum == theta) return SL_ERR_INVALID_ARG;
    return apply_coded(p, theta, momentum, mu, coded, coded_bytes, R, lr, stream);
}

int sl_payload_validate(sl_plan *p, const void *payload, void *workspace, void *stream)
{
    if (!p || !payload || !workspace) return SL_ERR_INVALID_ARG;
    if (misaligned(payload, 16) || misaligned(workspace, 256)) return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    return slk_validate(p, static_cast<const unsigned char *>(payload), static_cast<int *>(workspace),
                        static_cast<hipStream_t>(stream));
}

int sl_residual_apply(sl_plan *p, float *e, const void *payload, void *stream)
{
    if (!p || !e || !payload) return SL_ERR_INVALID_ARG;
    if (misaligned(e, 16) || misaligned(payload, 16)) return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    return slk_residual(p, e, static_cast<const unsigned char *>(payload),
                        static_cast<hipStream_t>(stream));
}

int sl_decompress_avg_apply(sl_plan *p, float *theta, const void *const *payloads, int R, float lr,
                            void *stream)
{
    if (!p || !theta || !payloads || R < 1 || R > SL_MAX_WORKERS) return SL_ERR_INVALID_ARG;
    if (misaligned(theta, 16)) return SL_ERR_INVALID_ARG;
    for (int r = 0; r < R; ++r)
        if (!payloads[r] || misaligned(payloads[r], 16)) return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    sl_prof_mark(p, -2, static_cast<hipStream_t>(stream));
    rc = slk_apply(p, theta, nullptr, 0.0f, payloads, R, lr, static_cast<hipStream_t>(stream));
    sl_prof_mark(p, SL_PROF_APPLY, static_cast<hipStream_t>(stream));
    return rc;
}

int sl_decompress_avg_apply_nesterov(sl_plan *p, float *theta, float *momentum, const void *const *payloads,
                                     int R, float lr, float mu, void *stream)
{
    if (!p || !theta || !momentum || theta == momentum || !payloads || R < 1 || R > SL_MAX_WORKERS)
        return SL_ERR_INVALID_ARG;
    if (misaligned(theta, 16) || misaligned(momentum, 16)) return SL_ERR_INVALID_ARG;
    for (int r = 0; r < R; ++r)
        if (!payloads[r] || misaligned(payloads[r], 16)) return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    sl_prof_mark(p, -2, static_cast<hipStream_t>(stream));
    rc = slk_apply(p, theta, momentum, mu, payloads, R, lr, static_cast<hipStream_t>(stream));
    sl_prof_mark(p, SL_PROF_APPLY, static_cast<hipStream_t>(stream));
    return rc;
}

int sl_lom_direction(sl_plan *p, float *m, const float *delta, float mu, float *dir, void *stream)
{
    if (!p || !m || !delta || !dir || m == delta || m == dir) return SL_ERR_INVALID_ARG;
    if (misaligned(m, 16) || misaligned(delta, 16) || misaligned(dir, 16)) return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    return slk_lom_direction(p, m, delta, mu, dir, static_cast<hipStream_t>(stream));
}

int sl_dense_avg_apply(sl_plan *p, float *theta, float *momentum, const float *const *dirs, int R, float lr,
                       float mu, void *stream)
{
    if (!p || !theta || theta == momentum || !dirs || R < 1 || R > SL_MAX_WORKERS) return SL_ERR_INVALID_ARG;
    if (misaligned(theta, 16) || misaligned(momentum, 16)) return SL_ERR_INVALID_ARG;
    for (int r = 0; r < R; ++r)
        if (!dirs[r] || dirs[r] == theta || dirs[r] == momentum || misaligned(dirs[r], 16))
            return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    return slk_dense_avg_apply(p, theta, momentum, dirs, R, lr, mu, static_cast<hipStream_t>(stream));
}

int sl_sub_topk(sl_plan *p, float *m, void *stream)
{
    if (!p || !m || misaligned(m, 16)) return SL_ERR_INVALID_ARG;
    int rc = check_device(p);
    if (rc) return rc;
    return slk_sub_topk(p, m, static_cast<hipStream_t>(stream));
}

int sl_pack_indices_bits(const uint16_t *idx, const uint8_t *codes, const float *values, int64_t n_chunks,
                         int k, int value_bits, void *out, void *stream)
{
    const int bits = value_bits;
    if (!(bits == 1 || bits == 2 || bits == 3 || bits == 4 || bits == 32)) return SL_ERR_INVALID_ARG;
    if (n_chunks < 0 || k < 4 || k > SL_CHUNK || (k & 3) || (bits != 2 && (k & 7))) return SL_ERR_INVALID_ARG;
    if (n_chunks > 0 && (!idx || !out || (bits == 32 ? !values : !codes))) return SL_ERR_INVALID_ARG;
    return slk_pack_bits(idx, codes, values, n_chunks, k, bits, static_cast<unsigned char *>(out),
                         static_cast<hipStream_t>(stream));
}

int sl_pack_indices(const uint16_t *idx, const uint8_t *codes, int64_t n_chunks, int k, void *out,
                    void *stream)
{
    if (n_chunks < 0 || k < 4 || k > SL_CHUNK || (k & 3)) return SL_ERR_INVALID_ARG;
    if (n_chunks > 0 && (!idx || !codes || !out)) return SL_ERR_INVALID_ARG;
    return slk_pack(idx, codes, n_chunks, k, static_cast<unsigned char *>(out),
                    static_cast<hipStream_t>(stream));
}

}  // extern "C"

// ---------------------------------------------------------------------------
// Optional per-kernel timing.  A compress call records up to 7 events (start + one after each
// of its phases), an apply call 2.
enum { PROF_CEV = 7 };
// event slot of a compress phase: 1 + phase, the coded format's placement passes last
static int prof_cslot(int phase) { return phase == SL_PROF_INDEX ? 6 : 1 + phase; }
static const int PROF_CPHASES[6] = {SL_PROF_SELECT, SL_PROF_STATS, SL_PROF_CODES, SL_PROF_LUT, SL_PROF_RESIDUAL,
                                    SL_PROF_INDEX};

struct SlProfile {
    int max_calls;
    int n_compress, n_apply;
    bool in_compress;
    std::vector<hipEvent_t> ev_compress;   // [max_calls][PROF_CEV]
    std::vector<hipEvent_t> ev_apply;      // [max_calls][2]
    std::vector<unsigned char> have;       // [max_calls][PROF_CEV] which compress events were recorded
    int cur;                               // slot of the call being recorded, or -1
};

void sl_prof_mark(const sl_plan *p, int phase, hipStream_t st)
{
    SlProfile *P = p->prof;
    if (!P) return;
    if (phase < 0) {               // start of a call: phase -1 = compress, -2 = apply
        P->in_compress = phase == -1;
        int &n = P->in_compress ? P->n_compress : P->n_apply;
        if (n >= P->max_calls) {
            P->cur = -1;
            return;
        }
        P->cur = n++;
        if (P->in_compress) {
            for (int i = 0; i < PROF_CEV; ++i) P->have[(size_t)P->cur * PROF_CEV + i] = 0;
            P->have[(size_t)P->cur * PROF_CEV] = 1;
            (void)hipEventRecord(P->ev_compress[(size_t)P->cur * PROF_CEV], st);
        } else {
            (void)hipEventRecord(P->ev_apply[(size_t)P->cur * 2], st);
        }
        return;
    }
    if (P->cur < 0) return;
    if (phase == SL_PROF_APPLY) {
        (void)hipEventRecord(P->ev_apply[(size_t)P->cur * 2 + 1], st);
    } else {
        P->have[(size_t)P->cur * PROF_CEV + prof_cslot(phase)] = 1;
        (void)hipEventRecord(P->ev_compress[(size_t)P->cur * PROF_CEV + prof_cslot(phase)], st);
    }
}

static void prof_free(SlProfile *P)
{
    if (!P) return;
    for (hipEvent_t e : P->ev_compress) (void)hipEventDestroy(e);
    for (hipEvent_t e : P->ev_apply) (void)hipEventDestroy(e);
    delete P;
}

extern "C" int sl_profile_begin(sl_plan *p, int max_calls)
{
    if (!p || max_calls < 1 || max_calls > 4096) return SL_ERR_INVALID_ARG;
    if (p->prof) {
        prof_free(p->prof);
        p->prof = nullptr;
    }
    SlProfile *P = new (std::nothrow) SlProfile();
    if (!P) return SL_ERR_NOMEM;
    P->max_calls = max_calls;
    P->n_compress = P->n_apply = 0;
    P->cur = -1;
    P->in_compress = false;
    try {
        P->have.assign((size_t)max_calls * PROF_CEV, 0);
        P->ev_compress.reserve((size_t)max_calls * PROF_CEV);
        P->ev_apply.reserve((size_t)max_calls * 2);
    } catch (const std::bad_alloc &) {
        delete P;
        return SL_ERR_NOMEM;
    }
    for (int i = 0; i < max_calls * PROF_CEV; ++i) {
        hipEvent_t e;
        hipError_t err = hipEventCreate(&e);
        if (err != hipSuccess) {
            prof_free(P);
            return hip_fail(err);
        }
        P->ev_compress.push_back(e);
    }
    for (int i = 0; i < max_calls * 2; ++i) {
        hipEvent_t e;
        hipError_t err = hipEventCreate(&e);
        if (err != hipSuccess) {
            prof_free(P);
            return hip_fail(err);
        }
        P->ev_apply.push_back(e);
    }
    p->prof = P;
    return SL_OK;
}

extern "C" int sl_profile_end(sl_plan *p, double *ms, int *calls)
{
    if (!p || !p->prof) return SL_ERR_INVALID_ARG;
    SlProfile *P = p->prof;
    double sum[SL_PROF_PHASES] = {0, 0, 0, 0, 0, 0, 0};
    int cnt[SL_PROF_PHASES] = {0, 0, 0, 0, 0, 0, 0};
    int rc = SL_OK;
    for (int c = 0; c < P->n_compress && rc == SL_OK; ++c) {
        int prev = 0;
        for (int i = 0; i < 6; ++i) {
            const int ph = PROF_CPHASES[i], slot = prof_cslot(ph);
            if (!P->have[(size_t)c * PROF_CEV + slot]) continue;
            hipEvent_t a = P->ev_compress[(size_t)c * PROF_CEV + prev], b = P->ev_compress[(size_t)c * PROF_CEV + slot];
            hipError_t err = hipEventSynchronize(b);
            float t = 0.f;
            if (err == hipSuccess) err = hipEventElapsedTime(&t, a, b);
            if (err != hipSuccess) {
                rc = hip_fail(err);
                break;
            }
            sum[ph] += t;
            cnt[ph]++;
            prev = slot;
        }
    }
    for (int c = 0; c < P->n_apply && rc == SL_OK; ++c) {
        hipError_t err = hipEventSynchronize(P->ev_apply[(size_t)c * 2 + 1]);
        float t = 0.f;
        if (err == hipSuccess)
            err = hipEventElapsedTime(&t, P->ev_apply[(size_t)c * 2], P->ev_apply[(size_t)c * 2 + 1]);
        if (err != hipSuccess) {
            rc = hip_fail(err);
            break;
        }
        sum[SL_PROF_APPLY] += t;
        cnt[SL_PROF_APPLY]++;
    }
    for (int ph = 0; ph < SL_PROF_PHASES; ++ph) {
        if (ms) ms[ph] = cnt[ph] ? sum[ph] / cnt[ph] : 0.0;
        if (calls) calls[ph] = cnt[ph];
    }
    prof_free(P);
    p->prof = nullptr;
    return rc;
}
