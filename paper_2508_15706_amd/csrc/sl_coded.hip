// Coded wire format: the passes that place the variable-length part (the chunks' quotient bit
// vectors), and the transcoder from a plain payload (sl_rice_encode).  The format is described
// in sl_coded.h; the appendix "Compression of indices in Top-k" of the paper is where an index
// coder enters the method.
//
// The writers of a coded buffer (kernel A of sl_compress_coded, or k_rice_chunks below for a
// payload that already exists) put everything whose place follows from the tensor list - table
// headers, remainder and value fields - straight into the buffer, and leave each chunk's bit
// vector and quotient sum Q in the workspace.  Then
//   k_coded_scan_tensor   one workgroup per tensor: words of each group's run, their exclusive
//                         prefix inside the tensor, the tensor's total;
//   k_coded_scan_list     one wave: prefix over the tensors, total size, buffer header;
//   k_coded_place         one wave per group: the 16 vectors shifted into one run, the run and
//                         the directory entry written.
#include "sl_coded.h"

int sl_rice_param(int k)
{
    const int q = 2839 / k;
    int b = 0;
    while ((2 << b) <= q) ++b;
    return q < 1 ? 0 : b;
}

namespace {

struct CodedArgs {
    SlCodedGeom G;
    const SlChunkDesc *desc;
    const SlTensorDev *tensors;
    const SlGroup *groups;
    long long n_groups, n_chunks;
    int n_tensors;
    const unsigned *uvec;           // [n_chunks][G.ua] bit vectors as the writers left them
    const unsigned short *qsum;     // [n_chunks]
    unsigned *gwords;               // [n_groups] words of each group's run
    unsigned *goff;                 // [n_groups] word offset of the run inside its tensor's part of the section
    unsigned long long *twords;     // [n_tensors + 1] words of each tensor's part, then (after the list scan) its offset
    unsigned char *out;             // the coded buffer
};

// Words of the run of the group that starts at chunk c0 of a tensor with n_chunks chunks.
SL_DEV unsigned group_words(const CodedArgs &A, const SlTensorDev &td, long long g)
{
    const long long c0 = g * SL_RICE_GROUP;
    const int nc = (int)min((long long)SL_RICE_GROUP, td.n_chunks - c0);
    unsigned bits = 0;
    for (int i = 0; i < nc; ++i) bits += (unsigned)A.G.k + A.qsum[td.chunk0 + c0 + i];
    return (bits + 31u) >> 5;
}

__global__ void __launch_bounds__(256) k_coded_scan_tensor(CodedArgs A)
{
    __shared__ unsigned long long wsum[4];
    __shared__ unsigned long long carry;
    const SlTensorDev td = A.tensors[blockIdx.x];
    const long long ng = (td.n_chunks + SL_RICE_GROUP - 1) / SL_RICE_GROUP;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = 0ull;
    __syncthreads();
    for (long long base = 0; base < ng; base += 256) {
        const long long i = base + tid;
        const unsigned v = i < ng ? group_words(A, td, i) : 0u;
        const unsigned incl = (unsigned)sl_wave_iscan((int)v);     // a tile's total stays far below 2^31
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        unsigned long long before = carry;
        for (int q = 0; q < wave; ++q) before += wsum[q];
        if (i < ng) {
            A.gwords[td.group0 + i] = v;
            A.goff[td.group0 + i] = (unsigned)(before + incl - v);
        }
        __syncthreads();
        if (tid == 255) carry = before + incl;
        __syncthreads();
    }
    if (tid == 0) A.twords[blockIdx.x] = carry;
}

// Prefix over the tensors (twords[t] becomes the tensor's offset in the section, in words), the
// buffer header, and the zero padding that rounds the buffer up to 16 bytes.
__global__ void __launch_bounds__(64) k_coded_scan_list(CodedArgs A)
{
    const int lane = threadIdx.x;
    unsigned long long pos = 0;
    for (int base = 0; base < A.n_tensors; base += 64) {
        const int t = base + lane;
        const unsigned long long v = t < A.n_tensors ? A.twords[t] : 0ull;
        unsigned long long incl = v;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const unsigned long long up = __shfl_up(incl, s);
            if (lane >= s) incl += up;
        }
        if (t < A.n_tensors) A.twords[t] = pos + incl - v;
        pos += __shfl(incl, 63);
    }
    const unsigned long long end = (unsigned long long)A.G.section + 4ull * pos;
    const unsigned long long total = (end + 15ull) & ~15ull;
    if (lane == 0) {
        unsigned long long *h = reinterpret_cast<unsigned long long *>(A.out);
        h[0] = 0x3230454349524C53ull;                      // "SLRICE02", little endian
        h[1] = total;
        A.twords[A.n_tensors] = pos;
    }
    if (end + 4ull * lane < total) *reinterpret_cast<unsigned *>(A.out + end + 4ull * lane) = 0u;
}

// One wave per group: its chunks' vectors, as the writers left them in the workspace (G.ua
// words each, bits beyond k + Q undefined), are shifted to their bit offsets inside the run
// in LDS; the run and the directory entry go to the buffer.
__global__ void __launch_bounds__(256) k_coded_place(CodedArgs A)
{
    extern __shared__ __align__(16) unsigned place_lds[];
    const int lane = threadIdx.x & 63;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long gi = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (gi >= A.n_groups) return;
    const SlCodedGeom &G = A.G;
    unsigned *run = place_lds + (size_t)wave * (SL_RICE_GROUP * G.ua + 1);
    const SlGroup g = A.groups[gi];
    const SlTensorDev td = A.tensors[g.tensor];
    const long long c0 = td.chunk0 + (long long)g.local_group * SL_RICE_GROUP;
    const int nc = (int)min((long long)SL_RICE_GROUP, td.n_chunks - (long long)g.local_group * SL_RICE_GROUP);
    const unsigned nw = A.gwords[gi];
    const unsigned long long base = A.twords[g.tensor] + A.goff[gi];    // below 2^32 by the plan's check

    const int q = lane < nc ? (int)A.qsum[c0 + lane] : 0;
    const int nbits = lane < nc ? G.k + q : 0;
    const int start = sl_wave_iscan(nbits) - nbits;                      // lanes 0..15 matter
    for (unsigned w = lane; w < nw + 1u; w += 64) run[w] = 0u;
    sl_wave_sync();
    for (int i = 0; i < nc; ++i) {
        const int s = __builtin_amdgcn_readlane(start, i), n = __builtin_amdgcn_readlane(nbits, i);
        const unsigned *src = A.uvec + (size_t)(c0 + i) * G.ua;
        const int words = (n + 31) >> 5, sh = s & 31;
        for (int j = lane; j < words; j += 64) {
            unsigned w = src[j];
            const int left = n - 32 * j;                                  // bits of this word that belong to the vector
            if (left < 32) w &= (1u << left) - 1u;
            sl_lds_or(&run[(s >> 5) + j], w << sh);
            if (sh) sl_lds_or(&run[(s >> 5) + j + 1], w >> (32 - sh));
        }
    }
    sl_wave_sync();
    unsigned *dst = reinterpret_cast<unsigned *>(A.out + G.section) + base;
    for (unsigned w = lane; w < nw; w += 64) dst[w] = run[w];
    unsigned char *entry = A.out + td.cdir_off + (long long)g.local_group * G.dent;
    if (lane == 0) *reinterpret_cast<unsigned *>(entry) = (unsigned)base;
    if (lane < SL_RICE_GROUP) {
        if (G.qf == 1) entry[4 + lane] = (unsigned char)q;
        else reinterpret_cast<unsigned short *>(entry + 4)[lane] = (unsigned short)q;
    }
}

// ------------------------------------------------------------------ transcoder, plain -> coded
// One wave per chunk: the record's 12-bit indices are unpacked into LDS and coded by the same
// routine as in kernel A of the compressor; the value fields and the table header are copied.
struct ChunksArgs {
    SlCodedGeom G;
    const SlChunkDesc *desc;
    const SlTensorDev *tensors;
    long long n_chunks;
    int rec_bytes;
    const unsigned char *payload;
    unsigned char *out;
    unsigned *uvec;
    unsigned short *qsum;
};

__global__ void __launch_bounds__(256) k_rice_chunks(ChunksArgs A)
{
    extern __shared__ __align__(16) unsigned char chunks_lds[];
    const int lane = threadIdx.x & 63;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= A.n_chunks) return;
    const SlCodedGeom &G = A.G;
    const int k = G.k, nrw = G.rem_bytes >> 2;
    const size_t per_wave = ((size_t)2 * k + 4 * ((size_t)G.ua + nrw) + 15) & ~(size_t)15;
    unsigned char *smem = chunks_lds + (size_t)wave * per_wave;
    unsigned *uv = reinterpret_cast<unsigned *>(smem);
    unsigned *rw = uv + G.ua;
    unsigned short *idx = reinterpret_cast<unsigned short *>(rw + nrw);
    const SlChunkDesc d = A.desc[c];
    const SlTensorDev td = A.tensors[d.tensor];
    const unsigned char *rec = A.payload + d.rec_off;
    for (int m = lane; m < k; m += 64) {
        const int b0 = (3 * m) >> 1;
        const unsigned w = (unsigned)rec[b0] | ((unsigned)rec[b0 + 1] << 8);
        idx[m] = (unsigned short)((m & 1) ? (w >> 4) : (w & 0xFFFu));
    }
    sl_wave_sync();
    const int Q = sl_coded_emit(G, lane, idx, uv, rw);
    unsigned char *fix = A.out + td.cfix_off + (long long)d.local_chunk * G.cfix;
    for (int w = lane; w < nrw; w += 64) reinterpret_cast<unsigned *>(fix)[w] = rw[w];
    // the value fields byte for byte, then the record's zero padding
    const unsigned char *vals = rec + 3 * k / 2;
    for (int i = lane; i < G.cfix - G.rem_bytes; i += 64) fix[G.rem_bytes + i] = i < G.val_bytes ? vals[i] : 0;
    unsigned *uvo = A.uvec + (size_t)c * G.ua;
    const int words = (k + Q + 31) >> 5;
    for (int w = lane; w < words; w += 64) uvo[w] = uv[w];
    if (lane == 0) A.qsum[c] = (unsigned short)Q;
    if (d.local_chunk == 0)                                        // the table header
        for (int i = lane; 4 * i < G.hdr; i += 64)
            reinterpret_cast<unsigned *>(A.out + td.cblk_off)[i] =
                reinterpret_cast<const unsigned *>(A.payload + td.pay_off)[i];
    if (d.local_chunk == td.n_chunks - 1) {                        // zero padding of the block
        const long long used = (td.cfix_off - td.cblk_off) + td.n_chunks * (long long)G.cfix;
        for (long long i = used + lane; i < td.cblk_bytes; i += 64) A.out[td.cblk_off + i] = 0;
    }
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

}  // namespace

// The passes that finish a coded buffer once its writers have run (see the top of this file).
int slk_coded_finish(const sl_plan *p, unsigned char *out, unsigned char *ws, hipStream_t st)
{
    CodedArgs A;
    A.G = p->cg;
    A.desc = p->d_desc;
    A.tensors = p->d_tensors;
    A.groups = p->d_groups;
    A.n_groups = p->n_groups;
    A.n_chunks = p->n_chunks;
    A.n_tensors = p->n_tensors;
    A.uvec = reinterpret_cast<const unsigned *>(ws + p->ws_uvec);
    A.qsum = reinterpret_cast<const unsigned short *>(ws + p->ws_qsum);
    A.gwords = reinterpret_cast<unsigned *>(ws + p->ws_gwords);
    A.goff = reinterpret_cast<unsigned *>(ws + p->ws_goff);
    A.twords = reinterpret_cast<unsigned long long *>(ws + p->ws_twords);
    A.out = out;
    int rc;
    if (p->n_groups > 0) {
        hipLaunchKernelGGL(k_coded_scan_tensor, dim3(p->n_tensors), dim3(256), 0, st, A);
        if ((rc = launched())) return rc;
    }
    hipLaunchKernelGGL(k_coded_scan_list, dim3(1), dim3(64), 0, st, A);
    if ((rc = launched())) return rc;
    if (p->n_groups > 0) {
        int wpb = 4;
        const size_t per_wave = ((size_t)SL_RICE_GROUP * p->cg.ua + 1) * sizeof(unsigned);
        while (wpb > 1 && per_wave * wpb > 65536) wpb >>= 1;
        hipLaunchKernelGGL(k_coded_place, dim3((unsigned)((p->n_groups + wpb - 1) / wpb)), dim3(64 * wpb),
                           per_wave * wpb, st, A);
        if ((rc = launched())) return rc;
    }
    return SL_OK;
}

int slk_rice_encode(const sl_plan *p, const unsigned char *payload, unsigned char *out,
                    unsigned char *ws, hipStream_t st)
{
    if (p->n_chunks > 0) {
        ChunksArgs C;
        C.G = p->cg;
        C.desc = p->d_desc;
        C.tensors = p->d_tensors;
        C.n_chunks = p->n_chunks;
        C.rec_bytes = p->rec_bytes;
        C.payload = payload;
        C.out = out;
        C.uvec = reinterpret_cast<unsigned *>(ws + p->ws_uvec);
        C.qsum = reinterpret_cast<unsigned short *>(ws + p->ws_qsum);
        const size_t per_wave = ((size_t)2 * p->k + 4 * ((size_t)p->cg.ua + (p->cg.rem_bytes >> 2)) + 15) & ~(size_t)15;
        hipLaunchKernelGGL(k_rice_chunks, dim3((unsigned)((p->n_chunks + 3) / 4)), dim3(256), per_wave * 4, st, C);
        const int rc = launched();
        if (rc) return rc;
    }
    return slk_coded_finish(p, out, ws, st);
}
