// The hot kernel: 1-bit weight bitlayers x activation bit planes by AND +
// population count (Sections 3.1 and 3.4 of the paper), plane weighting by
// [.., 2^1, 2^0] with a negative top plane (Algorithm 2) and scale-accumulation
// over the first `bits_used` bitlayers (Algorithm 2's loop; the run-time knob of
// the abstract), all in one launch.
//
// Mapping for CDNA4 (wave64):
//  * The activation planes are the small, endlessly reused operand: each wave
//    keeps the planes of its column slice in VGPRs for its whole life.  A quad
//    of 4 lanes owns 8 consecutive 32-bit column words; lane p of the quad owns
//    the planes 4t + p (t = pass).  The whole plane matrix of the slice is thus
//    spread over the 64 lanes with no copy held twice.
//  * Packed weight words stream from HBM exactly once, coalesced: a tile is
//    64 lanes x 2 words = 512 contiguous bytes per row chunk, loaded
//    non-temporally, kRing tiles in flight per wave.
//  * A lane needs the 8 weight words of its quad, not just its own 2: the
//    quad_perm DPP modifier on v_and_b32 broadcasts a neighbour's word for free,
//    so a (word, plane) pair costs exactly v_and_b32_dpp + v_bcnt_u32_b32 (the
//    popcount adds into its accumulator).
//  * Per tile a lane ends with one count per pass; v_mad_i32_i24 with per-lane
//    weights (+-2^j, split in a low and a high 16-plane half so that 32 bits
//    suffice) folds them into two integers.  The cross-lane sum of those is
//    deferred: 16 tiles are parked in LDS and reduced together.
//  * Planes that carry no information are skipped (see pb_prep.hip): the
//    kernel body is instantiated for 1..8 passes of 4 planes and picked at run
//    time from the statistics the prep kernel left in memory.
// All integer results are exact (int64 at the end), so they do not depend on
// the schedule.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "pb_kernels.h"

namespace pb {

struct MatvecArgs {
    const uint32_t *packed;
    const uint32_t *planes;
    const int *meta;
    const float *scales;
    float *Y;
    long long *A;
    size_t layer_words;
    size_t packed_bytes;
    int R, cwp, ws, rpt, csplit, rwaves;
    int m;               // bitlayers to accumulate
    int gw;              // row groups (tiles of rpt rows) per wave
    int num_rowgroups;   // rows_p / rpt
    int batch;
    int abuf_words;      // int64 slots per wave in the LDS result buffer
    double out_scale;    // 2^-frac_bits
};

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// One tile of packed weight words: raw buffer load, 8 bytes per lane, streaming (nt) so that
// words used once do not displace the planes in cache.  With the null descriptor (0 records)
// every lane is out of range: the load returns 0 and moves no data.
__device__ __forceinline__ uint2 load_tile(__amdgpu_buffer_rsrc_t rsrc, int voff, int soff)
{
    u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, voff, soff, /*nt*/ 2);
    return make_uint2(v.x, v.y);
}

// One pass over a tile: the lane's plane against the 8 weight words of its quad,
//   count = sum_n popcount(word_n & plane_word_n),
// as 8 x (v_and_b32 with the DPP quad broadcast riding on it + v_bcnt_u32_b32, which adds into its
// accumulator).  Word n of the quad lives in quad lane n / 2, component n % 2.  A single asm block keeps
// the 16 instructions back to back; the DPP source registers (w) come straight from a buffer load, never
// from a VALU write just before, so no DPP read-after-VALU-write wait states are needed.
#define PB_QP(Q) "quad_perm:[" #Q "," #Q "," #Q "," #Q "] row_mask:0xf bank_mask:0xf\n\t"
__device__ __forceinline__ uint32_t pass_count(const uint2 w, const uint32_t (&pl)[8])
{
    uint32_t acc, t;
    asm("v_and_b32_dpp %1, %2, %4 " PB_QP(0) "v_bcnt_u32_b32 %0, %1, 0\n\t"
        "v_and_b32_dpp %1, %3, %5 " PB_QP(0) "v_bcnt_u32_b32 %0, %1, %0\n\t"
        "v_and_b32_dpp %1, %2, %6 " PB_QP(1) "v_bcnt_u32_b32 %0, %1, %0\n\t"
        "v_and_b32_dpp %1, %3, %7 " PB_QP(1) "v_bcnt_u32_b32 %0, %1, %0\n\t"
        "v_and_b32_dpp %1, %2, %8 " PB_QP(2) "v_bcnt_u32_b32 %0, %1, %0\n\t"
        "v_and_b32_dpp %1, %3, %9 " PB_QP(2) "v_bcnt_u32_b32 %0, %1, %0\n\t"
        "v_and_b32_dpp %1, %2, %10 " PB_QP(3) "v_bcnt_u32_b32 %0, %1, %0\n\t"
        "v_and_b32_dpp %1, %3, %11 " PB_QP(3) "v_bcnt_u32_b32 %0, %1, %0"
        : "=&v"(acc), "=&v"(t)
        : "v"(w.x), "v"(w.y), "v"(pl[0]), "v"(pl[1]), "v"(pl[2]), "v"(pl[3]), "v"(pl[4]), "v"(pl[5]), "v"(pl[6]),
          "v"(pl[7]));
    return acc;
}
#undef PB_QP

// a * b + c for |a|, |b| < 2^23: a full-rate v_mad_i32_i24
__device__ __forceinline__ int mad24(int a, int b, int c) { return __mul24(a, b) + c; }

template <int NPASS>
__device__ __forceinline__ void tile_counts(const uint2 w, const uint32_t (&pr)[NPASS][8], const int (&mult)[8],
                                            int &lo, int &hi)
{
    lo = 0;
    hi = 0;
#pragma unroll
    for (int t = 0; t < NPASS; ++t) {
        const uint32_t acc = pass_count(w, pr[t]);
        if (t < 4) lo = mad24((int)acc, mult[t], lo);
        else hi = mad24((int)acc, mult[t], hi);
    }
}

// Per-wave constants shared by the prologue and the body.
struct WaveCtx {
    int lane, wave, slice, rw, n;
    int gbase, gcount, T;          // this wave's row groups and tile count (gcount * m)
    int voff;                      // this lane's byte offset inside a tile
    uint32_t soff;                 // byte offset of the next tile to load
    int ld_i, ld_t;                // bitlayer and index of the next tile to load
    uint32_t layer_bytes, wrap_bytes;
    __amdgpu_buffer_rsrc_t rs_data, rs_null;
};

__device__ __forceinline__ void issue_tile_load(WaveCtx &c, uint2 &dst, int m)
{
    dst = load_tile(c.ld_t < c.T ? c.rs_data : c.rs_null, c.voff, (int)c.soff);
    __builtin_amdgcn_sched_barrier(0x7);  // loads return in issue order: keep it the order of use
    ++c.ld_t;
    if (++c.ld_i == m) { c.ld_i = 0; c.soff += c.wrap_bytes; } else c.soff += c.layer_bytes;
}

// Planes of the wave's slice: lane (q, p) holds, for pass t, the 8 words of plane 4t + p that face its quad.
__device__ __forceinline__ void load_planes(const MatvecArgs &a, const WaveCtx &c, int t, uint32_t (&dst)[8])
{
    const int p = c.lane & 3, q = c.lane >> 2;
    const uint32_t *pl = a.planes + (size_t)c.n * 32 * (size_t)a.cwp;
    const int seg = c.slice * a.ws + ((q * 8) & (a.ws - 1));
    const uint4 *src = reinterpret_cast<const uint4 *>(pl + (size_t)(4 * t + p) * a.cwp + seg);
    uint4 v0 = src[0], v1 = src[1];
    dst[0] = v0.x; dst[1] = v0.y; dst[2] = v0.z; dst[3] = v0.w;
    dst[4] = v1.x; dst[5] = v1.y; dst[6] = v1.z; dst[7] = v1.w;
}

template <int NPASS, bool EARLY>
__device__ __forceinline__ void matvec_body(const MatvecArgs &a, WaveCtx &c, uint2 (&buf)[kRing], const int h,
                                            const float scv, const uint32_t (&pr_all)[8][8], char *smem)
{
    const int lane = c.lane, wave = c.wave, slice = c.slice, n = c.n;
    const int p = lane & 3;
    const int rpt = a.rpt, m = a.m;
    const int T = c.T, gbase = c.gbase, gcount = c.gcount;

    // LDS: per wave [kRing tiles][64 lanes] (lo, hi) pairs, then the int64 results of all waves
    int2 *red = reinterpret_cast<int2 *>(smem) + (size_t)wave * kRing * 64;
    long long *abuf_all = reinterpret_cast<long long *>(smem + (size_t)blockDim.x / 64 * kRing * 64 * sizeof(int2));
    long long *abuf = abuf_all + (size_t)wave * a.abuf_words;

    // --- planes of this wave's slice in registers; per-lane plane weights ---
    uint32_t pr[NPASS][8];
#pragma unroll
    for (int t = 0; t < NPASS; ++t) {
        if (EARLY) {
#pragma unroll
            for (int i = 0; i < 8; ++i) pr[t][i] = pr_all[t][i];
        } else {
            load_planes(a, c, t, pr[t]);
        }
    }
    if (!EARLY) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): planes (and the tiles issued before them) have landed
    int mult[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        int j = 4 * t + p;
        int wgt = 1 << (j & 15);
        mult[t] = (j < h) ? wgt : (j == h ? -wgt : 0);
    }

    // mapping of the deferred cross-lane sums: kRing * rpt outputs, 4 / rpt lanes each, 16 partials per lane
    const int lpo = 4 / rpt;
    const int o = lane / lpo;
    const int o_tile = o / rpt, o_row = o - o_tile * rpt;
    const int sub = lane - o * lpo;
    const int src0 = o_row * (64 / rpt) + sub * 16;

    for (int t0 = 0; t0 < T; t0 += kRing) {
#pragma unroll
        for (int u = 0; u < kRing; ++u) {
            if (t0 + u < T) {
                int lo, hi;
                tile_counts<NPASS>(buf[u], pr, mult, lo, hi);
                red[u * 64 + lane] = make_int2(lo, hi);
            }
            // the ring slot is free again: fetch the tile kRing ahead (a no-op load past the end)
            issue_tile_load(c, buf[u], m);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        {
            const int4 *rp = reinterpret_cast<const int4 *>(red + o_tile * 64 + src0);
            int lo = 0, hi = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int4 v = rp[(i + lane) & 7];
                lo += v.x + v.z;
                hi += v.y + v.w;
            }
            if (lpo >= 2) {
                lo += __builtin_amdgcn_mov_dpp(lo, 0xB1, 0xf, 0xf, true);
                hi += __builtin_amdgcn_mov_dpp(hi, 0xB1, 0xf, 0xf, true);
            }
            if (lpo == 4) {
                lo += __builtin_amdgcn_mov_dpp(lo, 0x4E, 0xf, 0xf, true);
                hi += __builtin_amdgcn_mov_dpp(hi, 0x4E, 0xf, 0xf, true);
            }
            if (sub == 0 && t0 + o_tile < T)
                abuf[(t0 + o_tile) * rpt + o_row] = (long long)lo + ((long long)hi << 16);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }

    // --- combine column slices, apply the layer scales, write ---
    if (a.csplit > 1) __syncthreads();
    if (slice == 0) {
        const int nout = gcount * rpt;
        for (int idx0 = 0; idx0 < nout; idx0 += 64) {
            const int idx = idx0 + lane;
            const int gl = idx / rpt, rr = idx - gl * rpt;
            const int row = (gbase + gl) * rpt + rr;
            const bool valid = idx < nout && row < a.R;
            double z = 0.0;
#pragma unroll
            for (int i = 0; i < PB_MAX_BITS; ++i) {
                if (i < m) {
                    const float si = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(scv), i));
                    if (valid) {
                        long long v = 0;
                        for (int s = 0; s < a.csplit; ++s)
                            v += abuf[(size_t)s * a.abuf_words + (gl * m + i) * rpt + rr];
                        if (a.A) a.A[((size_t)i * a.batch + n) * (size_t)a.R + row] = v;
                        else z += (double)si * (double)v;
                    }
                }
            }
            if (valid && !a.A) a.Y[(size_t)n * a.R + row] = (float)(z * a.out_scale);
        }
    }
}

// EARLY = fetch the planes of all 8 passes before anything else (no wait for the plane statistics; more cache
// traffic); otherwise only the passes in use are fetched, after the statistics arrive.
template <bool EARLY>
__global__ __launch_bounds__(512) void k_matvec(const MatvecArgs a)
{
    extern __shared__ __align__(16) char smem[];
    WaveCtx c;
    c.lane = threadIdx.x & 63;
    c.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    c.slice = c.wave % a.csplit;
    c.rw = c.wave / a.csplit;
    c.n = blockIdx.y;
    const int m = a.m;

    // scalar loads first: plane statistics and layer scales are needed late, their latency hides behind the tiles
    const int *mt = a.meta + (size_t)c.n * kMetaInts;
    const int h = mt[0];
    const int npass = mt[2];
    const float scv = a.scales ? a.scales[c.lane < m ? c.lane : m - 1] : 0.0f;  // lane i holds scales[i]

    // this wave's tiles: row groups [gbase, gbase + gcount), bitlayers [0, m); start the weight stream at once
    c.gbase = (blockIdx.x * a.rwaves + c.rw) * a.gw;
    int gcount = a.num_rowgroups - c.gbase;
    c.gcount = gcount < 0 ? 0 : (gcount > a.gw ? a.gw : gcount);
    c.T = c.gcount * m;
    c.voff = (int)(((c.lane * 2) / a.ws) * a.cwp + c.slice * a.ws + ((c.lane * 2) & (a.ws - 1))) * 4;
    const size_t rg_bytes = (size_t)a.rpt * (size_t)a.cwp * 4;
    const size_t base_off = (size_t)c.gbase * rg_bytes;
    const size_t avail = a.packed_bytes > base_off ? a.packed_bytes - base_off : 0;
    c.rs_data = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char *>(reinterpret_cast<const char *>(a.packed) + base_off), 0,
        (int)(avail > 0xFFFFFFFFull ? 0xFFFFFFFFull : avail), 0x00020000);
    c.rs_null = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(a.packed), 0, 0, 0x00020000);
    c.layer_bytes = (uint32_t)(a.layer_words * 4);
    c.wrap_bytes = (uint32_t)rg_bytes - (uint32_t)(m - 1) * c.layer_bytes;  // last layer -> next row group
    c.soff = 0;
    c.ld_i = 0;
    c.ld_t = 0;
    uint32_t pr_all[8][8];
    if (EARLY) {
#pragma unroll
        for (int t = 0; t < 8; ++t) load_planes(a, c, t, pr_all[t]);
        __builtin_amdgcn_sched_barrier(0x7);
    }
    uint2 buf[kRing];
#pragma unroll
    for (int u = 0; u < kRing; ++u) issue_tile_load(c, buf[u], m);

    switch (npass) {
        case 0: matvec_body<1, EARLY>(a, c, buf, h, scv, pr_all, smem); break;  // all-zero activations: the one pass weighs 0
        case 1: matvec_body<1, EARLY>(a, c, buf, h, scv, pr_all, smem); break;
        case 2: matvec_body<2, EARLY>(a, c, buf, h, scv, pr_all, smem); break;
        case 3: matvec_body<3, EARLY>(a, c, buf, h, scv, pr_all, smem); break;
        case 4: matvec_body<4, EARLY>(a, c, buf, h, scv, pr_all, smem); break;
        case 5: matvec_body<5, EARLY>(a, c, buf, h, scv, pr_all, smem); break;
        case 6: matvec_body<6, EARLY>(a, c, buf, h, scv, pr_all, smem); break;
        case 7: matvec_body<7, EARLY>(a, c, buf, h, scv, pr_all, smem); break;
        default: matvec_body<8, EARLY>(a, c, buf, h, scv, pr_all, smem); break;
    }
}

int launch_matvec(const uint32_t *packed, const float *scales, const Layout &L, int bits_used, int frac_bits,
                  const uint32_t *planes, const int *meta, int batch, float *Y, long long *A, hipStream_t st)
{
    MatvecArgs a;
    a.packed = packed; a.planes = planes; a.meta = meta; a.scales = scales; a.Y = Y; a.A = A;
    a.layer_words = L.layer_words;
    a.packed_bytes = packed_bytes(L);
    a.R = L.rows; a.cwp = L.cwp; a.ws = L.ws; a.rpt = L.rpt; a.csplit = L.csplit;
    a.rwaves = L.csplit == 1 ? 4 : (L.csplit == 2 ? 2 : (L.csplit <= 4 ? 2 : 1));
    int target_wgs = 512;
    bool early = false;
    if (const char *e = getenv("PB_TUNE_RWAVES")) a.rwaves = atoi(e);
    if (const char *e = getenv("PB_TUNE_WGS")) target_wgs = atoi(e);
    if (const char *e = getenv("PB_TUNE_EARLY")) early = atoi(e) != 0;
    if (a.csplit * a.rwaves > kMaxWavesPerWG) a.rwaves = 1;
    a.m = bits_used;
    a.num_rowgroups = L.rows_p / L.rpt;
    a.batch = batch;
    a.out_scale = ldexp(1.0, -frac_bits);
    // row groups per wave: aim at >= 2 workgroups per CU, bounded LDS result buffer
    long long per_wg = ((long long)a.num_rowgroups + target_wgs - 1) / target_wgs;
    int gw = (int)((per_wg + a.rwaves - 1) / a.rwaves);
    if (gw < 1) gw = 1;
    int gw_cap = 256 / (L.rpt * bits_used);
    if (gw_cap < 1) gw_cap = 1;
    if (gw > gw_cap) gw = gw_cap;
    a.gw = gw;
    a.abuf_words = gw * bits_used * L.rpt;
    const int waves = a.csplit * a.rwaves;
    long long nwg = ((long long)a.num_rowgroups + (long long)gw * a.rwaves - 1) / ((long long)gw * a.rwaves);
    size_t smem = (size_t)waves * kRing * 64 * sizeof(int2) + (size_t)waves * a.abuf_words * sizeof(long long);
    auto kern = early ? k_matvec<true> : k_matvec<false>;
    if (smem > 64 * 1024) {
        // more than the default 64 KB of dynamic LDS (a CU of this GPU has 160 KB)
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg, (unsigned)batch), dim3(waves * 64), smem, st, a);
    return (int)hipGetLastError();
}

}  // namespace pb
