// sl_decompress_avg_apply_coded: the aggregate + outer update (Algorithm 1, "Aggregate + Outer
// Update"; Eq. (2) lines 3-4) over R payloads in the CODED wire format (sl_coded.h; the
// appendix "Compression of indices in Top-k" is where the index coder enters the method), and
// sl_rice_decode, which uses the same decoder to write a plain payload.
//
// One wavefront owns one chunk, as in sl_apply.hip: fp32 accumulators of the chunk in LDS,
// workers added in the order r = 0..R-1, theta streamed through registers once.  What differs is
// how a worker's k (index, value) entries are found:
//   1. lane r reads worker r's directory entry: where the chunk's quotient bit vector lies;
//   2. the workers' fixed records (table, remainders, value fields) and bit vectors are staged
//      in LDS with coalesced loads, the first of them fetched ahead of the theta loads;
//   3. every lane takes one 32-bit word of some worker's vector and lists its zero bits: the
//      i-th zero of a vector, at bit z, ends entry i, whose quotients so far sum to z - i
//      (ranks from one prefix sum over the words' zero counts);
//   4. every lane takes 8 consecutive entries of some worker: their remainders are b bytes of
//      the record, a prefix sum over the lanes of a worker completes
//      idx_i = i + ((z_i - i) << b) + r_0 + ... + r_i, written back as 16-bit indices;
//   5. the additions, worker by worker, from those index lists.
// Steps 3 and 4 run for all workers of a batch at once, so their cost per chunk hardly grows
// with R; only step 5 is a chain over the workers.
#include "sl_coded.h"

namespace {

#ifndef SL_CAPPLY_STAGE
#define SL_CAPPLY_STAGE 4096      // LDS bytes for one batch of staged workers
#endif
#ifndef SL_CAPPLY_PFF
#define SL_CAPPLY_PFF 4           // words per lane fetched ahead of the theta loads: tables and fixed records,
#endif
#ifndef SL_CAPPLY_PFU
#define SL_CAPPLY_PFU 2           // ... bit vectors
#endif

struct CodedApplyArgs {
    SlCodedGeom G;
    const SlChunkDesc *desc;
    const SlCodedDesc *cdesc;
    const SlTensorDev *tensors;
    float *theta;
    float *mom;              // global outer momentum buffer (Nesterov variant), else null
    unsigned char *plain;    // MODE 2: the plain payload to write
    float mu, neg_lr, inv_R;
    int R;
    int batch;               // workers staged at a time
    int slot_bytes;          // LDS bytes of one staged worker
    int fwp;                 // words of (table header + fixed record)
    unsigned magic_l;        // floor(2^32 / d) + 1 for d = lanes per worker in step 4
    int lpw_log2;            // staging: log2 of the lanes that fetch one worker's words (64 / lanes >= batch)
    int uwp_log2;            // log2 of the slots per worker in step 3 (a power of two >= G.ua)
    int E;                   // entries per lane in step 4: 8, or 4 when k is not a multiple of 8
    int rec_bytes;           // MODE 2: bytes of a plain record
    int lds_per_wave;
    long long n_chunks;
    const unsigned char *payload[SL_MAX_WORKERS];
    unsigned sec_words[SL_MAX_WORKERS];   // words of each payload's quotient section
};

SL_DEV void acc_add(float *acc, unsigned j, float q) { acc[j] = acc[j] + q; }

// MODE 0: theta update; 1: with DiLoCo's global Nesterov momentum (Eq. (1)); 2: no update at
// all - the one payload is decoded into a plain payload (R = 1).
template <bool TWO_BIT, int MODE>
__global__ void __launch_bounds__(256) k_apply_coded(CodedApplyArgs A)
{
    constexpr bool NESTEROV = MODE == 1, DECODE = MODE == 2;
    extern __shared__ __align__(16) unsigned char smem_all[];
    const SlCodedGeom &G = A.G;
    const int lane = threadIdx.x & 63, k = G.k, b = G.b;
    const int wave = sl_uniform((int)(threadIdx.x >> 6));
    const long long c = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (c >= A.n_chunks) return;
    unsigned char *smem = smem_all + (size_t)wave * A.lds_per_wave;
    float *acc = reinterpret_cast<float *>(smem);
    unsigned char *stage = smem + (DECODE ? 0 : SL_CHUNK * sizeof(float));
    const SlChunkDesc d = A.desc[c];
    const SlCodedDesc cd = A.cdesc[c];
    const int bits = TWO_BIT ? 2 : G.bits;
    const int hdr = TWO_BIT ? 16 : G.hdr, hdrw = hdr >> 2;
    const int fwp = A.fwp, uraw = G.ua + 1;
    // one staged worker: [table header][fixed record][uraw words of the bit vector][k 16-bit values]
    const int off_u = 4 * fwp, off_h = (off_u + 4 * uraw + 15) & ~15;

    float *tc = DECODE ? nullptr : A.theta + d.base;
    const int lr = lane >> 4, lc = (lane & 15) * 4;
    const unsigned stride = (unsigned)d.stride;
    const bool full = d.flags & SLC_FULL;

    // lane l keeps worker l's payload pointer and section size; the others read them across lanes
    static_assert(SL_MAX_WORKERS <= 64, "one payload per lane");
    const unsigned long long my_ptr = reinterpret_cast<unsigned long long>(A.payload[lane]);
    const unsigned my_words = A.sec_words[lane];
    asm volatile("" ::"v"(my_words));   // arrives with the pointer: no later wait may count it among the prefetches
    auto payload_of = [&](int r) -> sl_gbytes {
        const unsigned lo = (unsigned)sl_lane_read((int)(unsigned)my_ptr, r);
        const unsigned hi = (unsigned)sl_lane_read((int)(unsigned)(my_ptr >> 32), r);
        return reinterpret_cast<sl_gbytes>(((unsigned long long)hi << 32) | lo);
    };
    // Step 1, once for all workers: lane r < R learns where worker r keeps the chunk's bit vector:
    // first word (bounded by the section's size when it is used), shift and length.  This is the one
    // load that the loads of the vectors depend on.
    unsigned v_word = 0;         // first word of the vector, from the start of the section
    int v_meta = k << 5;         // (first bit inside that word) | (bits << 5)
    if (lane < A.R) {
        const SlVecPlace P = sl_coded_dir_entry(G, reinterpret_cast<sl_gbytes>(my_ptr) + cd.dir_off, cd.pos);
        v_word = P.run_word + (unsigned)(P.start_bit >> 5);
        v_meta = (P.start_bit & 31) | (P.nbits << 5);
    }
    // Staging.  A batch's workers share the wave's lanes: lanes [rs * LPW, (rs + 1) * LPW) fetch the words
    // of the batch's worker rs, LPW words at a time, so a lane needs its worker's pointer, vector place and
    // section size once per batch (four lane reads) and its addresses step by a constant.  Two parts per
    // worker, each fetched by straight-line code: fwp words of (table header, fixed record) and uraw words
    // of the bit vector (all ones beyond a payload's end: no entries).
    const int LPW = 1 << A.lpw_log2, rs = lane >> A.lpw_log2, qs = lane & (LPW - 1);
    unsigned char *const my_stage = stage + rs * A.slot_bytes;
    struct StageSrc {
        sl_gbytes p;
        unsigned word0, limit;
        bool live;
    };
    auto stage_src = [&](int r0, int nb) -> StageSrc {
        StageSrc S;
        S.live = rs < nb;
        const int r = S.live ? r0 + rs : r0;
        S.p = payload_of(r);
        S.word0 = (unsigned)sl_lane_read((int)v_word, r);
        S.limit = (unsigned)sl_lane_read((int)my_words, r);
        return S;
    };
    auto src_fixed = [&](const StageSrc &S, int u) -> unsigned {
        const int q = qs + (u << A.lpw_log2);
        const bool valid = S.live && q < fwp;
        const long long at = q < hdrw ? cd.lut_off + 4 * q : cd.fix_off + 4 * (q - hdrw);
        return valid ? *reinterpret_cast<sl_gwords>(S.p + at) : 0u;
    };
    auto src_vector = [&](const StageSrc &S, int u) -> unsigned {
        const int q = qs + (u << A.lpw_log2);
        const unsigned long long at = (unsigned long long)S.word0 + (unsigned)q;
        return (S.live && q < uraw && at < S.limit) ? reinterpret_cast<sl_gwords>(S.p + G.section)[at] : 0xFFFFFFFFu;
    };
    auto park_fixed = [&](int nb, int u, unsigned v) {
        const int q = qs + (u << A.lpw_log2);
        if (rs < nb && q < fwp) reinterpret_cast<unsigned *>(my_stage)[q] = v;
    };
    auto park_vector = [&](int nb, int u, unsigned v) {
        const int q = qs + (u << A.lpw_log2);
        if (rs < nb && q < uraw) reinterpret_cast<unsigned *>(my_stage + off_u)[q] = v;
    };

    constexpr int PFF = SL_CAPPLY_PFF, PFU = SL_CAPPLY_PFU;
    unsigned pf_f[PFF], pf_u[PFU], pn_f[PFF], pn_u[PFU];
    const int nb0 = min(A.batch, A.R);

    sl_f4 th[DECODE ? 1 : 16], mo[NESTEROV ? 16 : 1];
    float *mc = NESTEROV ? A.mom + d.base : nullptr;
    // The first 64 * PF words of the first batch are fetched BEFORE the theta loads: loads complete in
    // order, so the decode then waits for these few words only and runs while the chunk's 16 KB of
    // theta are in flight.  (Tried: the directory entry one chunk ahead, a wave taking several chunks
    // in turn - the loop costs more registers than a wave has next to a second one; and half of the
    // theta loads ahead of these words, which leaves too little of the stream behind the decode.)
    {
        const StageSrc S = stage_src(0, nb0);
#pragma unroll
        for (int u = 0; u < PFF; ++u) pf_f[u] = src_fixed(S, u);
#pragma unroll
        for (int u = 0; u < PFU; ++u) pf_u[u] = src_vector(S, u);
    }
    if constexpr (!DECODE) {
        // Sixteen loads are issued for EVERY chunk, so that the wait in front of the words fetched above
        // is "all but the last sixteen" whatever the chunk: a ragged chunk (a tensor's edge) reads its own
        // descriptor sixteen times instead, and then loads its elements one by one, without branches (an
        // element outside the chunk reads the chunk's first one and is replaced by zero).  Were the
        // sixteen under a condition, the number of loads behind those words would be unknown and the
        // wait would be for all of them on the full chunks too.
        {
            const float *none = reinterpret_cast<const float *>(A.desc + c);
            const float *ts = full ? tc : none, *ms = (NESTEROV && full) ? mc : none;
            const unsigned o0 = full ? 4u * (lr * stride + lc) : 0u, step = full ? 16u * stride : 0u;
#pragma unroll
            for (int i = 0; i < 16; ++i) th[i] = sl_load_stream_at(ts, i * step, o0);
            if constexpr (NESTEROV) {
#pragma unroll
                for (int i = 0; i < 16; ++i) mo[i] = sl_load_stream_at(ms, i * step, o0);
            }
        }
        if (!full) {
            const int rows = d.rows, cols = d.cols, last_cols = d.last_cols;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = 4 * i + lr;
                const int lim = row < rows - 1 ? cols : (row == rows - 1 ? last_cols : 0);
                const unsigned o0 = row * stride + lc;
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    const bool in = lc + cc < lim;
                    const unsigned at = in ? o0 + cc : 0u;
                    const float tv = __builtin_nontemporal_load(tc + at);
                    th[i][cc] = in ? tv : 0.f;
                    if constexpr (NESTEROV) {
                        const float mv = __builtin_nontemporal_load(mc + at);
                        mo[i][cc] = in ? mv : 0.f;
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
            reinterpret_cast<float4 *>(acc)[i * 64 + lane] = make_float4(0.f, 0.f, 0.f, 0.f);
    }

    const int E = A.E, L = k / E;                 // step 4: entries per lane, lanes per worker
    const int uwp = 1 << A.uwp_log2;
    // One batch of workers: staged, decoded, added.  The first batch is processed by straight-line code
    // of its own ahead of the loop over the others: inside a loop the wait in front of the staged words
    // is for every outstanding load, the theta loads included, and the decode would start only once the
    // whole chunk has arrived; ahead of the loop it is for the words alone.
    auto do_batch = [&](const int r0, const bool first) __attribute__((always_inline)) {
        const int nb = min(A.batch, A.R - r0);
        sl_wave_sync();
        // ---- step 2: stage the batch.  The first words of both parts are in registers: fetched ahead of
        // the theta loads for the first batch (pf_*), while the previous batch was decoded for the others
        // (pn_*: registers of their own, so that the wait in front of the first batch's words stays
        // "everything but the theta loads" - one array written on both paths would make it "everything").
        {
            if (first) {
#pragma unroll
                for (int u = 0; u < PFF; ++u) park_fixed(nb, u, pf_f[u]);
#pragma unroll
                for (int u = 0; u < PFU; ++u) park_vector(nb, u, pf_u[u]);
            } else {
#pragma unroll
                for (int u = 0; u < PFF; ++u) park_fixed(nb, u, pn_f[u]);
#pragma unroll
                for (int u = 0; u < PFU; ++u) park_vector(nb, u, pn_u[u]);
            }
            if ((PFF << A.lpw_log2) < fwp || (PFU << A.lpw_log2) < uraw) {      // what the registers did not hold
                const StageSrc S = stage_src(r0, nb);
                for (int u = PFF; (u << A.lpw_log2) < fwp; u += 2) {
                    const unsigned v0 = src_fixed(S, u), v1 = src_fixed(S, u + 1);
                    park_fixed(nb, u, v0);
                    park_fixed(nb, u + 1, v1);
                }
                for (int u = PFU; (u << A.lpw_log2) < uraw; u += 2) {
                    const unsigned v0 = src_vector(S, u), v1 = src_vector(S, u + 1);
                    park_vector(nb, u, v0);
                    park_vector(nb, u + 1, v1);
                }
                // (every load of this block has been waited for by a lane that parked its word; said once
                // more for all of them, so that the registers they used are not taken to be in flight by
                // code that follows - which would put a wait for the theta loads in front of steps 4 and 5
                // on the lists that never come here)
                __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
            }
            if (r0 + A.batch < A.R) {
                const StageSrc S = stage_src(r0 + A.batch, min(A.batch, A.R - r0 - A.batch));
#pragma unroll
                for (int u = 0; u < PFF; ++u) pn_f[u] = src_fixed(S, u);
#pragma unroll
                for (int u = 0; u < PFU; ++u) pn_u[u] = src_vector(S, u);
            }
            sl_wave_sync();
        }
        // the dequantised value of a staged worker's entry m
        auto value_at = [&](const unsigned char *slot, int m) -> float {
            const float *lutp = reinterpret_cast<const float *>(slot);
            const unsigned char *vals = slot + 4 * hdrw + G.rem_bytes;
            if (TWO_BIT) return lutp[(vals[m >> 2] >> (2 * (m & 3))) & 3u];
            if (bits == 32) return reinterpret_cast<const float *>(vals)[m];
            return lutp[sl_code_at(vals, m, bits)];
        };
        // ---- no remainders (b = 0, k above 1419): a gap is its quotient, the vector is the chunk's bit map -
        // bit p is zero exactly where index p is selected - and the entries are added straight from it, the
        // i-th zero with the i-th value, worker after worker.  (Steps 3 to 5 would give the same sums.)
        if (!DECODE && b == 0) {
            const int passes = (G.ua + 63) >> 6;
            for (int r = 0; r < nb; ++r) {
                const unsigned char *slot = stage + r * A.slot_bytes;
                const unsigned *raw = reinterpret_cast<const unsigned *>(slot + off_u);
                const int meta = sl_lane_read(v_meta, r0 + r);
                const int sh = meta & 31, n = meta >> 5;
                int carry = 0;
                for (int t = 0; t < passes; ++t) {
                    const int j = 64 * t + lane;
                    unsigned zeros = 0;
                    if (j < G.ua) {
                        const unsigned w = __builtin_amdgcn_alignbit(raw[j + 1], raw[j], (unsigned)sh);
                        const int left = n - 32 * j;
                        const unsigned mask = left >= 32 ? 0xFFFFFFFFu : left > 0 ? (1u << left) - 1u : 0u;
                        zeros = ~w & mask;
                    }
                    const int nz = __builtin_popcount(zeros);
                    const int incl = sl_wave_iscan(nz);
                    int lo = carry + incl - nz, hi = lo + nz - 1;    // entries of the word's lowest and highest zero
                    carry += __builtin_amdgcn_readlane(incl, 63);
                    // Two zeros per turn, one from each end of the word: two independent chains, their LDS
                    // reads issued together.  (An entry beyond k - 1 can only come from a malformed vector
                    // and takes the last entry's value.)
                    if constexpr (TWO_BIT) {
                        // the word's nz two-bit codes, entry `lo` at bit 0 of a 64-bit window
                        const unsigned *cw = reinterpret_cast<const unsigned *>(slot + 4 * hdrw + G.rem_bytes);
                        const int e0 = min(lo, k - 1), wi = (2 * e0) >> 5, csh = (2 * e0) & 31;
                        const unsigned c0 = cw[wi], c1 = cw[wi + 1], c2 = cw[wi + 2];
                        unsigned long long wl = ((unsigned long long)__builtin_amdgcn_alignbit(c2, c1, (unsigned)csh) << 32) |
                                                __builtin_amdgcn_alignbit(c1, c0, (unsigned)csh);
                        unsigned long long wh = nz ? wl << (64 - 2 * nz) : 0ull;      // entry `hi` in the two top bits
                        const float *lutp = reinterpret_cast<const float *>(slot);
                        while (zeros) {
                            const int pl = __builtin_ctz(zeros), ph = 31 - __builtin_clz(zeros);
                            const float q_lo = lutp[(unsigned)wl & 3u], q_hi = lutp[(unsigned)(wh >> 62)];
                            const unsigned j_lo = (unsigned)(32 * j + pl), j_hi = (unsigned)(32 * j + ph);
                            const float a_lo = acc[j_lo], a_hi = acc[j_hi];
                            acc[j_lo] = a_lo + q_lo;
                            if (ph != pl) acc[j_hi] = a_hi + q_hi;
                            zeros &= zeros - 1u;
                            zeros &= ~(1u << ph);
                            wl >>= 2, wh <<= 2;
                        }
                    } else {
                        while (zeros) {
                            const int pl = __builtin_ctz(zeros), ph = 31 - __builtin_clz(zeros);
                            const float q_lo = value_at(slot, min(lo, k - 1));
                            const float q_hi = value_at(slot, min(hi, k - 1));
                            acc_add(acc, (unsigned)(32 * j + pl), q_lo);
                            if (ph != pl) acc_add(acc, (unsigned)(32 * j + ph), q_hi);
                            zeros &= zeros - 1u;
                            zeros &= ~(1u << ph);
                            ++lo, --hi;
                        }
                    }
                }
                sl_wave_sync();               // worker r is complete before worker r+1 is added
            }
            return;
        }
        // ---- step 3: the zero bits of the vectors -> running quotient sums, by entry
        {
            const int slots = nb << A.uwp_log2;
            int carry = 0;
            for (int s0 = 0; s0 < slots; s0 += 64) {
                const int slot = s0 + lane;
                const int r = slot >> A.uwp_log2, j = slot & (uwp - 1);
                const bool live = slot < slots && j < G.ua;
                const int meta = sl_lane_read(v_meta, live ? r0 + r : 0);
                const int sh = meta & 31, n = meta >> 5;
                unsigned zeros = 0;
                unsigned short *hs = reinterpret_cast<unsigned short *>(stage + (live ? r : 0) * A.slot_bytes + off_h);
                if (live) {
                    const unsigned *raw = reinterpret_cast<const unsigned *>(stage + r * A.slot_bytes + off_u);
                    const unsigned w = __builtin_amdgcn_alignbit(raw[j + 1], raw[j], (unsigned)sh);
                    const int left = n - 32 * j;
                    const unsigned mask = left >= 32 ? 0xFFFFFFFFu : left > 0 ? (1u << left) - 1u : 0u;
                    zeros = ~w & mask;
                }
                const int nz = __builtin_popcount(zeros);
                const int incl = sl_wave_iscan(nz);
                int rank;
                if (uwp <= 64) {
                    const int seg = lane & ~(uwp - 1);                 // first lane of this worker's words
                    const int before = sl_lane_read(incl, seg > 0 ? seg - 1 : 0);
                    rank = incl - nz - (seg > 0 ? before : 0);
                } else {
                    if ((s0 & (uwp - 1)) == 0) carry = 0;              // a new worker starts with this pass
                    rank = carry + incl - nz;
                    carry += __builtin_amdgcn_readlane(incl, 63);
                }
                // The word's zero bits, two from each end per turn of the loop (four independent chains; the
                // length of this loop - the word with the most zeros - is on the chunk's critical path).  Entry
                // `rank` is the word's lowest zero, entry `rank + nz - 1` its highest; when one zero is left both
                // ends write the same value to the same place.  A vector with more than k zeros (malformed)
                // takes the loop that checks every store.
                if (__builtin_amdgcn_ballot_w64(rank + nz > k) == 0) {
                    // (byte addresses and values as plain integers the compiler may not take apart again:
                    // it would rebuild each of them from j and rank in every turn)
                    unsigned lo = (unsigned)(size_t)(hs + rank), hi = (unsigned)(size_t)(hs + rank + nz - 1);
                    int vlo = 32 * j - rank, vhi = 32 * j + 31 - (rank + nz - 1);
                    asm volatile("" : "+v"(lo), "+v"(hi), "+v"(vlo), "+v"(vhi));
                    auto put = [](unsigned at, int v) {
                        *reinterpret_cast<unsigned short __attribute__((address_space(3))) *>(at) = (unsigned short)v;
                    };
                    while (zeros) {
                        const int pl = __builtin_ctz(zeros), ch = __builtin_clz(zeros);
                        put(lo, vlo + pl);
                        put(hi, vhi - ch);
                        zeros &= (zeros - 1u) & ~(0x80000000u >> ch);
                        if (zeros) {
                            const int pl2 = __builtin_ctz(zeros), ch2 = __builtin_clz(zeros);
                            put(lo + 2, vlo - 1 + pl2);
                            put(hi - 2, vhi + 1 - ch2);
                            zeros &= (zeros - 1u) & ~(0x80000000u >> ch2);
                        }
                        lo += 4, hi -= 4, vlo -= 2, vhi += 2;
                    }
                } else {
                    int rk = rank;
                    while (zeros) {
                        const int pl = __builtin_ctz(zeros);
                        if (rk < k) hs[rk] = (unsigned short)(32 * j + pl - rk);
                        zeros &= zeros - 1u;
                        ++rk;
                    }
                }
            }
            sl_wave_sync();
        }
        // ---- step 4: remainders, their prefix sums, the indices
        {
            const int wpp = L <= 64 ? 64 / L : 1;       // workers per pass
            const int ppw = (L + 63) >> 6;              // passes per worker (1 unless L > 64)
            const unsigned fmask = (1u << b) - 1u;
            for (int rb = 0; rb < nb; rb += wpp) {
                int carry = 0;
                for (int ps = 0; ps < ppw; ++ps) {
                    // (lane / L; the multiplier does not exist for L = 1)
                    const int rl = L == 1 ? lane : L <= 64 ? (int)__umulhi((unsigned)lane, A.magic_l) : 0;
                    const int o = L <= 64 ? lane - rl * L : 64 * ps + lane;
                    const int r = rb + rl;
                    const bool live = rl < wpp && r < nb && o < L;
                    unsigned char *slot = stage + (live ? r : 0) * A.slot_bytes;
                    int pre[8];
                    int total = 0;
                    if (live) {
                        // (the two words behind the one that holds the first field are read whether or not
                        // the fields reach them: they lie inside the worker's slot)
                        const unsigned *rem = reinterpret_cast<const unsigned *>(slot + 4 * hdrw);
                        const int bit = o * E * b, wi = bit >> 5;
                        const unsigned w0 = rem[wi], w1 = rem[wi + 1], w2 = rem[wi + 2];
                        const unsigned lo = __builtin_amdgcn_alignbit(w1, w0, (unsigned)(bit & 31));
                        const unsigned hi = __builtin_amdgcn_alignbit(w2, w1, (unsigned)(bit & 31));
                        const unsigned long long win = ((unsigned long long)hi << 32) | lo;
                        int t = 0;
                        if (b <= 8) {
                            // four fields fit a word: entries 0..3 from the window's low word, 4..7 from
                            // the word that starts at field 4
                            const unsigned lo4 = (unsigned)(win >> (4 * b));
#pragma unroll
                            for (int e = 0; e < 4; ++e) pre[e] = (t += (int)__builtin_amdgcn_ubfe(lo, (unsigned)(e * b), (unsigned)b));
#pragma unroll
                            for (int e = 0; e < 4; ++e) pre[4 + e] = (t += (int)__builtin_amdgcn_ubfe(lo4, (unsigned)(e * b), (unsigned)b));
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e) pre[e] = (t += (int)((unsigned)(win >> (e * b)) & fmask));
                        }
                        total = E == 8 ? pre[7] : pre[3];
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) pre[e] = 0;
                    }
                    const int incl = sl_wave_iscan(total);
                    int excl;
                    if (L <= 64) {
                        const int seg = rl * L;
                        const int before = sl_lane_read(incl, seg > 0 ? seg - 1 : 0);
                        excl = incl - total - (seg > 0 ? before : 0);
                    } else {
                        excl = carry + incl - total;
                        carry += __builtin_amdgcn_readlane(incl, 63);
                    }
                    if (live) {
                        unsigned short *hs = reinterpret_cast<unsigned short *>(slot + off_h) + o * E;
                        unsigned short hv[8];
                        if (E == 8) {
                            const uint4 q4 = *reinterpret_cast<const uint4 *>(hs);
                            hv[0] = (unsigned short)q4.x, hv[1] = (unsigned short)(q4.x >> 16);
                            hv[2] = (unsigned short)q4.y, hv[3] = (unsigned short)(q4.y >> 16);
                            hv[4] = (unsigned short)q4.z, hv[5] = (unsigned short)(q4.z >> 16);
                            hv[6] = (unsigned short)q4.w, hv[7] = (unsigned short)(q4.w >> 16);
                        } else {
                            const uint2 q2 = *reinterpret_cast<const uint2 *>(hs);
                            hv[0] = (unsigned short)q2.x, hv[1] = (unsigned short)(q2.x >> 16);
                            hv[2] = (unsigned short)q2.y, hv[3] = (unsigned short)(q2.y >> 16);
                            hv[4] = hv[5] = hv[6] = hv[7] = 0;
                        }
                        // two indices per word, cut to 12 bits each after packing: a malformed payload stays
                        // inside the chunk (a valid one never reaches bit 12)
                        unsigned pw[4];
                        const unsigned base = (unsigned)(o * E) + (unsigned)excl;
#pragma unroll
                        for (int e = 0; e < 8; e += 2) {
                            const unsigned i0 = base + (unsigned)e + ((unsigned)hv[e] << b) + (unsigned)pre[e];
                            const unsigned i1 = base + (unsigned)(e + 1) + ((unsigned)hv[e + 1] << b) + (unsigned)pre[e + 1];
                            pw[e >> 1] = (i0 | (i1 << 16)) & 0x0FFF0FFFu;
                        }
                        if (E == 8)
                            *reinterpret_cast<uint4 *>(hs) = make_uint4(pw[0], pw[1], pw[2], pw[3]);
                        else
                            *reinterpret_cast<uint2 *>(hs) = make_uint2(pw[0], pw[1]);
                    }
                }
            }
            sl_wave_sync();
        }
        if constexpr (DECODE) {
            // ---- plain record: the 12-bit index stream, then the value fields byte for byte
            const unsigned short *idx = reinterpret_cast<const unsigned short *>(stage + off_h);
            unsigned char *rec = A.plain + d.rec_off;
            const int nbytes = 3 * k / 2;
            for (int q = lane; q < nbytes; q += 64) {
                const int bit0 = 8 * q, m = bit0 / 12, sh = bit0 - 12 * m;     // 0, 4 or 8
                unsigned v = (unsigned)idx[m] >> sh;
                if (sh == 8 && m + 1 < k) v |= (unsigned)idx[m + 1] << 4;
                rec[q] = (unsigned char)v;
            }
            const unsigned char *vals = stage + 4 * hdrw + G.rem_bytes;
            for (int q = lane; q < G.val_bytes; q += 64) rec[nbytes + q] = vals[q];
            if (d.local_chunk == 0 || d.local_chunk == A.tensors[d.tensor].n_chunks - 1) {
                const SlTensorDev td = A.tensors[d.tensor];
                if (d.local_chunk == 0)
                    for (int q = lane; q < hdrw; q += 64)
                        reinterpret_cast<unsigned *>(A.plain + td.pay_off)[q] = reinterpret_cast<const unsigned *>(stage)[q];
                if (d.local_chunk == td.n_chunks - 1)
                    for (long long q = hdr + td.n_chunks * (long long)A.rec_bytes + lane; q < td.block_bytes; q += 64)
                        A.plain[td.pay_off + q] = 0;
            }
        } else {
            // ---- step 5: the additions, worker by worker
            if (k <= 128) {
                // the entries of up to eight workers are fetched first (independent LDS reads),
                // then added worker by worker: the additions form a chain of LDS round trips
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
                            if (rb + u < nb && m < k) {
                                const unsigned char *slot = stage + (rb + u) * A.slot_bytes;
                                jj[u][s2] = reinterpret_cast<const unsigned short *>(slot + off_h)[m];
                                qq[u][s2] = value_at(slot, m);
                            }
                        }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        if (rb + u < nb) {
#pragma unroll
                            for (int s2 = 0; s2 < 2; ++s2)
                                if (jj[u][s2] != 0xFFFFu) acc_add(acc, jj[u][s2], qq[u][s2]);
                            sl_wave_sync();   // worker r is complete before worker r+1 is added
                        }
                    }
                }
            } else {
                // four consecutive entries per lane: one 8-byte read of indices, the positions of one
                // record are distinct, so the four reads and the four writes are issued together
                for (int r = 0; r < nb; ++r) {
                    const unsigned char *slot = stage + r * A.slot_bytes;
                    const unsigned short *idx = reinterpret_cast<const unsigned short *>(slot + off_h);
                    for (int q4 = lane; q4 < (k >> 2); q4 += 64) {
                        const uint2 iw = *reinterpret_cast<const uint2 *>(idx + 4 * q4);
                        const unsigned j0 = iw.x & 0xFFFFu, j1 = iw.x >> 16, j2 = iw.y & 0xFFFFu, j3 = iw.y >> 16;
                        const float q0 = value_at(slot, 4 * q4), q1 = value_at(slot, 4 * q4 + 1),
                                    q2 = value_at(slot, 4 * q4 + 2), q3 = value_at(slot, 4 * q4 + 3);
                        const float t0 = acc[j0], t1 = acc[j1], t2 = acc[j2], t3 = acc[j3];
                        acc[j0] = t0 + q0, acc[j1] = t1 + q1, acc[j2] = t2 + q2, acc[j3] = t3 + q3;
                    }
                    sl_wave_sync();           // worker r is complete before worker r+1 is added
                }
            }
        }
    };
    do_batch(0, true);
    for (int r0 = A.batch; r0 < A.R; r0 += A.batch) do_batch(r0, false);

    if constexpr (!DECODE) {
        if (full) {
            const unsigned o0 = 4u * (lr * stride + lc), step = 16u * stride;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float4 a = reinterpret_cast<const float4 *>(acc)[i * 64 + lane];
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
            for (int i = 0; i < 16; ++i) {
                const int row = 4 * i + lr;
                const int lim = row < rows - 1 ? cols : (row == rows - 1 ? last_cols : 0);
                const unsigned o0 = row * stride + lc;
                const float4 a = reinterpret_cast<const float4 *>(acc)[i * 64 + lane];
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

int pow2_log2_at_least(int n)
{
    int l = 0;
    while ((1 << l) < n) ++l;
    return l;
}

}  // namespace

// mode 0: theta update; 1: with the global momentum `mom`; 2: decode payloads[0] into `plain`.
int slk_apply_coded(const sl_plan *p, int mode, float *theta, float *mom, float mu, unsigned char *plain,
                    const void *const *payloads, const size_t *bytes, int R, float lr, hipStream_t st)
{
    if (p->n_chunks == 0) return SL_OK;
    CodedApplyArgs A;
    A.G = p->cg;
    A.desc = p->d_desc;
    A.cdesc = p->d_cdesc;
    A.tensors = p->d_tensors;
    A.theta = theta;
    A.mom = mom;
    A.plain = plain;
    A.mu = mu;
    A.neg_lr = -lr;
    A.inv_R = 1.0f / (float)R;
    A.R = R;
    const SlCodedGeom &G = p->cg;
    A.fwp = (G.hdr + G.cfix) >> 2;
    A.E = (G.k & 7) ? 4 : 8;
    A.rec_bytes = p->rec_bytes;
    A.slot_bytes = (int)(((((size_t)4 * A.fwp + 4 * ((size_t)G.ua + 1) + 15) & ~(size_t)15) + 2 * (size_t)G.k + 15) & ~(size_t)15);
    A.uwp_log2 = pow2_log2_at_least(G.ua);
    int batch = SL_CAPPLY_STAGE / A.slot_bytes;
    // (a whole number of passes of step 3, where a pass holds several workers' vectors)
    const int per_pass = A.uwp_log2 < 6 ? 64 >> A.uwp_log2 : 1;
    if (batch > per_pass) batch -= batch % per_pass;
    if (batch < 1) batch = 1;
    if (batch > R) batch = R;
    A.batch = batch;
    A.lpw_log2 = 6 - pow2_log2_at_least(batch);
    const int L = G.k / A.E;
    A.magic_l = L > 1 ? (unsigned)(0x100000000ull / (unsigned)L + 1) : 0u;
    A.n_chunks = p->n_chunks;
    for (int r = 0; r < SL_MAX_WORKERS; ++r) {
        A.payload[r] = r < R ? static_cast<const unsigned char *>(payloads[r]) : nullptr;
        const size_t sec = r < R && bytes[r] > (size_t)G.section ? (bytes[r] - (size_t)G.section) >> 2 : 0;
        A.sec_words[r] = sec > 0xFFFFFFFFull ? 0xFFFFFFFFu : (unsigned)sec;
    }
    A.lds_per_wave = (int)(((mode == 2 ? 0 : SL_CHUNK * sizeof(float)) + (size_t)batch * A.slot_bytes + 15) & ~(size_t)15);
    int wpb = 4;
    while (wpb > 1 && (size_t)A.lds_per_wave * wpb > (size_t)p->max_lds) wpb >>= 1;
    const size_t lds = (size_t)A.lds_per_wave * wpb;
    typedef void (*kernel_t)(CodedApplyArgs);
    static const kernel_t table[2][3] = {{k_apply_coded<false, 0>, k_apply_coded<false, 1>, k_apply_coded<false, 2>},
                                         {k_apply_coded<true, 0>, k_apply_coded<true, 1>, k_apply_coded<true, 2>}};
    const kernel_t fn = table[p->bits == 2 ? 1 : 0][mode];
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
