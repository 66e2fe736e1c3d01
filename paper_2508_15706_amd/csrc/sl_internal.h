// Internal structures shared by the host API and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sparseloco.h"

// One 4096-element chunk seen as a 64-row view: element (row, col) of the view
// is arena[base + row*stride + col].  A FLAT chunk is the view with stride 64.
// `rows` valid rows; every valid row has `cols` valid columns except the last
// valid row, which has `last_cols`.  Everything a kernel needs to know about a
// chunk comes with one 32-byte scalar load.
struct SlChunkDesc {
    long long base;
    int stride;
    unsigned char rows, cols, last_cols, flags;
    long long rec_off;      // byte offset of the chunk's record inside a payload
    int tensor;             // index of the tensor in the list
    int local_chunk;        // index of the chunk inside its tensor
};
static_assert(sizeof(SlChunkDesc) == 32, "descriptor is one 32-byte load");
enum { SLC_FULL = 1 };   // all 4096 positions valid (rows need not be 16-byte aligned)

struct SlTensorDev {
    long long chunk0;       // first chunk of the tensor in list order
    long long n_chunks;
    long long pay_off;      // byte offset of the tensor's block in a payload
    long long block_bytes;  // align16(16 + n_chunks * record_bytes)
    long long group0;       // first directory group (16 chunks) of the tensor, list order
    // coded format: byte offsets inside a coded buffer of the tensor's block (table header first),
    // of its directory and of its first fixed record; size of the block
    long long cblk_off, cdir_off, cfix_off, cblk_bytes;
};

enum { SL_RICE_GROUP = 16 };  // chunks per directory entry of the coded format

// Where a chunk's parts lie in a coded buffer (byte offsets that follow from the tensor list):
// what the coded aggregate needs about a chunk besides its SlChunkDesc, in one 32-byte load.
struct SlCodedDesc {
    long long lut_off;      // table header of the chunk's tensor block
    long long dir_off;      // directory entry of the chunk's group
    long long fix_off;      // the chunk's fixed record
    int pos;                // position of the chunk in its group, 0..15
    int reserved;
};
static_assert(sizeof(SlCodedDesc) == 32, "descriptor is one 32-byte load");

// Sizes of the coded format that follow from k and the value width (see sl_coded.h).
struct SlCodedGeom {
    int k, bits;
    int b;                  // Rice parameter
    int qmax;               // largest possible sum of a chunk's quotients, (4096 - k) >> b
    int qf;                 // bytes of a quotient-sum field in the directory: 1 or 2
    int dent;               // bytes of a directory entry: 4 + 16 * qf
    int rem_bytes;          // the k remainders, padded to 4 bytes
    int val_bytes;          // the k value fields: k * bits / 8
    int cfix;               // fixed record: rem_bytes + val_bytes padded to 4
    int hdr;                // table header of a tensor block
    int ua;                 // words of a chunk's longest bit vector: ceil((k + qmax) / 32)
    long long section;      // byte offset of the quotient section (end of the last block)
};

struct SlGroup {            // one coding group of the index coder
    int tensor;
    int local_group;
};

// Per-tensor quantizer state produced during sl_compress.
struct SlTensorStat {
    double mu;      // mean of the selected values
    double var;     // their population variance (bin edges sit at multiples of sigma)
};
static_assert(sizeof(SlTensorStat) == 16, "");

// Sizes of the wire format for `bits` value bits (1..4, or 32 = unquantized
// fp32 values): look-up table header of a tensor block and one chunk record.
__host__ __device__ inline int sl_hdr_bytes(int bits)
{
    return bits == 32 ? 0 : ((4 << bits) < 16 ? 16 : (4 << bits));
}
__host__ __device__ inline int sl_rec_bytes(int k, int bits) { return 3 * k / 2 + k * bits / 8; }

// Code of entry m in a little-endian stream of `bits`-wide fields (bits <= 4).
__host__ __device__ inline unsigned sl_code_at(const unsigned char *codes, int m, int bits)
{
    const int bit = m * bits, sh = bit & 7;
    unsigned w = codes[bit >> 3];
    if (sh + bits > 8) w |= (unsigned)codes[(bit >> 3) + 1] << 8;
    return (w >> sh) & ((1u << bits) - 1u);
}

struct sl_plan {
    int k;
    int bits;                   // value bits: 1..4, or 32 for unquantized fp32 values
    int rec_bytes, hdr_bytes;   // sl_rec_bytes(k, bits), sl_hdr_bytes(bits)
    int n_tensors;
    int device;
    int max_lds;                // largest LDS allocation of one workgroup, bytes
    int64_t n_chunks;
    int64_t n_elements;
    int64_t n_partial;          // chunks without SLC_FULL
    size_t payload_bytes;
    size_t ws_bytes;
    // workspace sections (byte offsets)
    size_t ws_vals, ws_leafA, ws_leafC, ws_cnt, ws_tstat;
    // device tables
    SlChunkDesc *d_desc;
    SlCodedDesc *d_cdesc;
    SlTensorDev *d_tensors;
    SlGroup *d_groups;
    int64_t n_groups;
    size_t rice_max_bytes;      // upper bound of a coded buffer, 0 when the list is beyond the coded format
    SlCodedGeom cg;
    // workspace sections of the coded path: per-chunk bit vectors (cg.ua words each) and quotient
    // sums, per-group run lengths and offsets (words), per-tensor section offsets (words)
    size_t ws_uvec, ws_qsum, ws_gwords, ws_goff, ws_twords;
    long long codes_wave_below; // list length below which the code kernel gives a chunk to a wave at any k
    // host copies
    SlTensorDev *h_tensors;
    // optional per-kernel timing (sl_profile_begin / sl_profile_end)
    struct SlProfile *prof;
};

// Byte offset of the LUT header of the chunk's tensor block inside a payload.
__host__ __device__ inline long long sl_lut_off(const SlChunkDesc &d, int hdr_bytes, int rec_bytes)
{
    return d.rec_off - hdr_bytes - (long long)d.local_chunk * rec_bytes;
}

// Records an event after the kernel of `phase` (phase < 0: start of a call).
void sl_prof_mark(const sl_plan *p, int phase, hipStream_t st);

// sl_compress and its variants behind one argument check (sl_api.hip)
// (coded != null: the coded wire format is written as well, `coded_capacity` bytes available)
int sl_compress_impl(sl_plan *p, float *e, const float *delta, const float *theta_local, float beta,
                     int flags, const void *pending, void *payload, void *workspace, void *stream,
                     bool random = false, unsigned seed = 0u, void *coded = nullptr, size_t coded_capacity = 0);

// device address of the library's own scratch array on `device` (the current device), sl_noalloc.hip
int sl_noalloc_scratch(int device, void **out);

// launchers (defined next to their kernels)
int slk_select(const sl_plan *p, float *e, const float *delta, const float *theta_local, float beta,
               int frozen, const unsigned char *pending, unsigned char *payload, unsigned char *coded,
               unsigned char *ws, hipStream_t st);
// the same with Random-k in place of Top-k
int slk_select_random(const sl_plan *p, float *e, const float *delta, float beta, int frozen,
                      const unsigned char *pending, unsigned char *payload, unsigned char *ws, unsigned seed,
                      hipStream_t st);
// B, C, D and (unless skip_residual) E
int slk_quantize(const sl_plan *p, float *e, int skip_residual, unsigned char *payload, unsigned char *coded,
                 unsigned char *ws, hipStream_t st);
// E on its own: e[idx] -= LUT[code] for the entries of `payload`
int slk_residual(const sl_plan *p, float *e, const unsigned char *payload, hipStream_t st);
// mom != null: DiLoCo's global Nesterov momentum on top of the aggregate
int slk_apply(const sl_plan *p, float *theta, float *mom, float mu, const void *const *payloads, int R,
              float lr, hipStream_t st);
// dense outer steps of the DiLoCo family (sl_outer.hip) and Sub-k (sl_select.hip)
int slk_lom_direction(const sl_plan *p, float *m, const float *delta, float mu, float *dir, hipStream_t st);
int slk_dense_avg_apply(const sl_plan *p, float *theta, float *mom, const float *const *dirs, int R, float lr,
                        float mu, hipStream_t st);
int slk_sub_topk(const sl_plan *p, float *m, hipStream_t st);
int slk_validate(const sl_plan *p, const unsigned char *payload, int *flag, hipStream_t st);
int slk_pack(const uint16_t *idx, const uint8_t *codes, int64_t n_chunks, int k, unsigned char *out,
             hipStream_t st);
int slk_pack_bits(const uint16_t *idx, const uint8_t *codes, const float *values, int64_t n_chunks, int k,
                  int bits, unsigned char *out, hipStream_t st);
int slk_rice_encode(const sl_plan *p, const unsigned char *payload, unsigned char *out,
                    unsigned char *ws, hipStream_t st);
// coded wire format: the passes that place the quotient bit vectors once a buffer's writers have run
int slk_coded_finish(const sl_plan *p, unsigned char *out, unsigned char *ws, hipStream_t st);
// mode 0: theta update from R coded payloads; 1: with the global momentum `mom`; 2: payloads[0] decoded into `plain`
int slk_apply_coded(const sl_plan *p, int mode, float *theta, float *mom, float mu, unsigned char *plain,
                    const void *const *payloads, const size_t *bytes, int R, float lr, hipStream_t st);
int sl_rice_param(int k);
void sl_note_hip_error(hipError_t e);
