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
//    64 lanes x 2 words = 512 contiguous bytes per row chunk, fetched with
//    non-temporal raw buffer loads, kRing tiles in flight per wave.
//  * A lane needs the 8 weight words of its quad, not just its own 2: eight
//    v_mov_b32 with the quad_perm DPP modifier broadcast them once per tile;
//    every (word, plane) pair then costs one v_and_b32 (a double-rate VOP2 on
//    this chip) and one v_bcnt_u32_b32, which adds into its accumulator.
//  * Per tile a lane ends with one count per pass; v_mad_i32_i24 with per-lane
//    weights (+-2^j, split in a low and a high 16-plane half so that 32 bits
//    suffice) folds them into two integers.  The cross-lane sum of those is
//    deferred: kRing tiles are parked in LDS and reduced together.
//  * Planes that carry no information are skipped (see pb_prep.hip): the
//    kernel body is instantiated for 1..8 passes of 4 planes and picked at run
//    time from the statistics the prep kernel left in memory.  The first
//    kSpecPasses passes are fetched before those statistics arrive (one memory
//    round trip less on the critical path), the rest only if needed.
// All integer results are exact (int64 at the end), so they do not depend on
// the schedule.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "pb_kernels.h"

namespace pb {

constexpr int kRedTiles = kRing;  // tiles whose per-lane partial sums are parked in LDS and reduced together
constexpr int kSpecPasses = 5;   // passes (of 4 planes) fetched speculatively: 20 planes cover N(0,1) * 2^16

struct MatvecArgs {
    const uint32_t *packed;
    const uint32_t *planes;
    const int *meta;
    const float *scales;
    float *Y;
    long long *A;
    size_t layer_words;
    size_t packed_bytes;
    int R, cwp, ws, ws_shift, rpt, rpt_shift, csplit, csplit_magic, rwaves;
    int m;               // bitlayers to accumulate
    int gw;              // row groups (tiles of rpt rows) per wave
    int num_rowgroups;   // rows_p / rpt
    int batch;
    int abuf_words;      // (lo, hi) slots per wave in the LDS result buffer
    double out_scale;    // 2^-frac_bits
};

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// count = sum_n popcount(bw[n] & plane[n]) over the 8 column words of the lane's quad: 8 x (v_and_b32 +
// v_bcnt_u32_b32, which adds into its accumulator), two accumulators so that no instruction waits for the
// one before it.  The asm keeps the popcounts a chain of accumulating v_bcnt (the compiler would rebuild
// them as a tree of separate adds).
__device__ __forceinline__ uint32_t pass_count(const uint32_t (&bw)[8], const uint32_t (&pl)[8])
{
    uint32_t a0, a1, t0, t1;
    asm("v_and_b32 %2, %4, %12\n\t"
        "v_and_b32 %3, %5, %13\n\t"
        "v_bcnt_u32_b32 %0, %2, 0\n\t"
        "v_bcnt_u32_b32 %1, %3, 0\n\t"
        "v_and_b32 %2, %6, %14\n\t"
        "v_and_b32 %3, %7, %15\n\t"
        "v_bcnt_u32_b32 %0, %2, %0\n\t"
        "v_bcnt_u32_b32 %1, %3, %1\n\t"
        "v_and_b32 %2, %8, %16\n\t"
        "v_and_b32 %3, %9, %17\n\t"
        "v_bcnt_u32_b32 %0, %2, %0\n\t"
        "v_bcnt_u32_b32 %1, %3, %1\n\t"
        "v_and_b32 %2, %10, %18\n\t"
        "v_and_b32 %3, %11, %19\n\t"
        "v_bcnt_u32_b32 %0, %2, %0\n\t"
        "v_bcnt_u32_b32 %1, %3, %1\n\t"
        "v_add_u32 %0, %0, %1"
        : "=&v"(a0), "=&v"(a1), "=&v"(t0), "=&v"(t1)
        : "v"(bw[0]), "v"(bw[1]), "v"(bw[2]), "v"(bw[3]), "v"(bw[4]), "v"(bw[5]), "v"(bw[6]), "v"(bw[7]),
          "v"(pl[0]), "v"(pl[1]), "v"(pl[2]), "v"(pl[3]), "v"(pl[4]), "v"(pl[5]), "v"(pl[6]), "v"(pl[7]));
    return a0;
}

template <int Q>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, Q * 0x55, 0xf, 0xf, true);
}

// a * b + c for |a|, |b| < 2^23: v_mad_i32_i24
__device__ __forceinline__ int mad24(int a, int b, int c) { return __mul24(a, b) + c; }

template <int NPASS>
__device__ __forceinline__ void tile_counts(const uint2 w, const uint32_t (&pr)[8][8], const int (&mult)[8], int &lo,
                                            int &hi)
{
    // word n of the quad lives in quad lane n / 2, component n % 2
    uint32_t bw[8];
    bw[0] = quad_bcast<0>(w.x); bw[1] = quad_bcast<0>(w.y);
    bw[2] = quad_bcast<1>(w.x); bw[3] = quad_bcast<1>(w.y);
    bw[4] = quad_bcast<2>(w.x); bw[5] = quad_bcast<2>(w.y);
    bw[6] = quad_bcast<3>(w.x); bw[7] = quad_bcast<3>(w.y);
    lo = 0;
    hi = 0;
#pragma unroll
    for (int t = 0; t < NPASS; ++t) {
        const uint32_t cnt = pass_count(bw, pr[t]);
        if (t < 4) lo = mad24((int)cnt, mult[t], lo);
        else hi = mad24((int)cnt, mult[t], hi);
    }
}

// Per-wave state of the weight stream.
struct Stream {
    const char *base;              // first tile of this wave
    uint32_t avail;                // bytes from base to the end of the packed array
    int voff;                      // this lane's byte offset inside a tile
    uint32_t soff;                 // byte offset of the next tile to load
    int ld_i, ld_t, T, m;          // bitlayer / index of the next tile, tile count, bitlayers
    uint32_t layer_bytes, wrap_bytes;
};

// One tile of packed weight words: raw buffer load, 8 bytes per lane, streaming (nt) so that words used once
// do not displace the planes in cache.  Past the last tile the descriptor has 0 records: every lane is out of
// range, the load returns 0 and moves no data.  Loads return in issue order, so the issue order is kept the
// order of use (the sched_barrier lets only ALU instructions move across).
__device__ __forceinline__ void issue_tile_load(Stream &s, uint2 &dst)
{
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(s.base), 0, s.ld_t < s.T ? (int)s.avail : 0, 0x00020000);
    u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rs, s.voff, (int)s.soff, /*nt*/ 2);
    dst = make_uint2(v.x, v.y);
    __builtin_amdgcn_sched_barrier(0x7);
    ++s.ld_t;
    if (++s.ld_i == s.m) { s.ld_i = 0; s.soff += s.wrap_bytes; } else s.soff += s.layer_bytes;
}

// Planes of the wave's slice: lane (q, p) holds, for pass t, the 8 words of plane 4t + p that face its quad.
__device__ __forceinline__ void load_planes(const uint32_t *lane_planes, int cwp, int t, uint32_t (&dst)[8])
{
    const uint4 *src = reinterpret_cast<const uint4 *>(lane_planes + (size_t)(4 * t) * cwp);
    uint4 v0 = src[0], v1 = src[1];
    dst[0] = v0.x; dst[1] = v0.y; dst[2] = v0.z; dst[3] = v0.w;
    dst[4] = v1.x; dst[5] = v1.y; dst[6] = v1.z; dst[7] = v1.w;
}

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int NPASS>
__device__ __forceinline__ void matvec_body(const MatvecArgs &a, Stream &s, uint2 (&buf)[kRing],
                                            const uint32_t (&pr)[8][8], const int (&mult)[8], int2 *red, int2 *abuf,
                                            int lane)
{
    const int rpt = a.rpt, rs = a.rpt_shift, T = s.T;
    // mapping of the deferred cross-lane sums: kRedTiles * rpt outputs, 8 / rpt lanes each, 8 partials per lane
    const int lpo_shift = 3 - rs;
    const int o = lane >> lpo_shift;
    const int o_tile = o >> rs, o_row = o & (rpt - 1);
    const int sub = lane & ((1 << lpo_shift) - 1);
    const int src0 = o_row * (64 >> rs) + sub * 8;
    const int4 *rp = reinterpret_cast<const int4 *>(red + o_tile * 64 + src0);

    for (int t0 = 0; t0 < T; t0 += kRedTiles) {
#pragma unroll
        for (int u = 0; u < kRedTiles; ++u) {
            if (t0 + u < T) {
                int lo, hi;
                tile_counts<NPASS>(buf[u], pr, mult, lo, hi);
                red[u * 64 + lane] = make_int2(lo, hi);
            }
            // the ring slot is free again: fetch the tile kRing ahead (a no-op load past the end).  Issued
            // unconditionally so that the number of loads in flight is the same on every path.
            issue_tile_load(s, buf[u]);
        }
        wave_lds_sync();
        int lo = 0, hi = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int4 v = rp[(i + lane) & 3];
            lo += v.x + v.z;
            hi += v.y + v.w;
        }
        lo += __builtin_amdgcn_mov_dpp(lo, 0xB1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
        hi += __builtin_amdgcn_mov_dpp(hi, 0xB1, 0xf, 0xf, true);
        if (lpo_shift >= 2) {
            lo += __builtin_amdgcn_mov_dpp(lo, 0x4E, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
            hi += __builtin_amdgcn_mov_dpp(hi, 0x4E, 0xf, 0xf, true);
        }
        if (lpo_shift == 3) {
            lo += __builtin_amdgcn_mov_dpp(lo, 0x141, 0xf, 0xf, true);  // row_half_mirror: the other quad of the 8
            hi += __builtin_amdgcn_mov_dpp(hi, 0x141, 0xf, 0xf, true);
        }
        if (sub == 0 && t0 + o_tile < T) abuf[((t0 + o_tile) << rs) + o_row] = make_int2(lo, hi);
        wave_lds_sync();
    }
}

__global__ __launch_bounds__(512) void k_matvec(const MatvecArgs a)
{
    extern __shared__ __align__(16) char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rw = (wave * a.csplit_magic) >> 16;   // wave / csplit
    const int slice = wave - rw * a.csplit;
    const int n = blockIdx.y;
    const int m = a.m;
    const int p = lane & 3, q = lane >> 2;

    // plane statistics and layer scales: issued first, needed late
    // (a vector load: a scalar load would make every later wait for kernel arguments wait for it too)
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const __amdgpu_buffer_rsrc_t rs_meta = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int *>(a.meta + (size_t)n * kMetaInts), 0, kMetaInts * 4, 0x00020000);
    const i32x4 mv = __builtin_amdgcn_raw_buffer_load_b128(rs_meta, 0, 0, 0);
    const float scv = a.scales ? a.scales[lane < m ? lane : m - 1] : 0.0f;  // lane i holds scales[i]

    // planes of the first passes, then this wave's weight tiles: row groups [gbase, gbase + gcount), layers [0, m)
    const int seg = slice * a.ws + ((q * 8) & (a.ws - 1));
    const uint32_t *lane_planes = a.planes + ((size_t)n * 32 + p) * (size_t)a.cwp + seg;
    uint32_t pr[8][8];
#pragma unroll
    for (int t = 0; t < kSpecPasses; ++t) load_planes(lane_planes, a.cwp, t, pr[t]);
    __builtin_amdgcn_sched_barrier(0x7);

    const int gbase = (blockIdx.x * a.rwaves + rw) * a.gw;
    int gcount = a.num_rowgroups - gbase;
    gcount = gcount < 0 ? 0 : (gcount > a.gw ? a.gw : gcount);
    Stream s;
    s.T = gcount * m;
    s.m = m;
    s.voff = (int)((((lane * 2) >> a.ws_shift) * a.cwp + slice * a.ws + ((lane * 2) & (a.ws - 1))) * 4);
    const size_t rg_bytes = (size_t)a.rpt * (size_t)a.cwp * 4;
    const size_t base_off = (size_t)gbase * rg_bytes;
    s.base = reinterpret_cast<const char *>(a.packed) + base_off;
    s.avail = (uint32_t)(a.packed_bytes > base_off ? a.packed_bytes - base_off : 0);
    s.layer_bytes = (uint32_t)(a.layer_words * 4);
    s.wrap_bytes = (uint32_t)rg_bytes - (uint32_t)(m - 1) * s.layer_bytes;  // last layer -> next row group
    s.soff = 0;
    s.ld_i = 0;
    s.ld_t = 0;
    uint2 buf[kRing];
#pragma unroll
    for (int u = 0; u < kRing; ++u) issue_tile_load(s, buf[u]);

    // the statistics are here by now: remaining passes (rare), per-lane plane weights
    const int h = __builtin_amdgcn_readfirstlane(mv.x);
    const int npass = __builtin_amdgcn_readfirstlane(mv.z);
    if (npass > kSpecPasses) {
#pragma unroll
        for (int t = kSpecPasses; t < 8; ++t)
            if (t < npass) load_planes(lane_planes, a.cwp, t, pr[t]);
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing older than the steady-state tile loads stays pending
    }
    int mult[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int j = 4 * t + p;
        const int wgt = 1 << (j & 15);
        mult[t] = (j < h) ? wgt : (j == h ? -wgt : 0);   // planes above h repeat the sign plane: together -2^h
    }

    // LDS: per wave [kRedTiles][64 lanes] (lo, hi) pairs, then the per-(tile, row) sums of all waves
    const int nwaves = blockDim.x >> 6;
    int2 *red = reinterpret_cast<int2 *>(smem) + (size_t)wave * kRedTiles * 64;
    int2 *abuf = reinterpret_cast<int2 *>(smem + (size_t)nwaves * kRedTiles * 64 * sizeof(int2)) +
                 (size_t)wave * a.abuf_words;

    switch (npass) {
        case 0:  // all-zero activations: the one pass weighs 0
        case 1: matvec_body<1>(a, s, buf, pr, mult, red, abuf, lane); break;
        case 2: matvec_body<2>(a, s, buf, pr, mult, red, abuf, lane); break;
        case 3: matvec_body<3>(a, s, buf, pr, mult, red, abuf, lane); break;
        case 4: matvec_body<4>(a, s, buf, pr, mult, red, abuf, lane); break;
        case 5: matvec_body<5>(a, s, buf, pr, mult, red, abuf, lane); break;
        case 6: matvec_body<6>(a, s, buf, pr, mult, red, abuf, lane); break;
        case 7: matvec_body<7>(a, s, buf, pr, mult, red, abuf, lane); break;
        default: matvec_body<8>(a, s, buf, pr, mult, red, abuf, lane); break;
    }

    // --- combine column slices, apply the layer scales, write: one lane per output row ---
    // A_i = lo + hi * 2^16 exactly (both halves are int32), so fp64(A_i) = fp64(lo) + fp64(hi) * 65536 exactly.
    if (a.csplit > 1) __syncthreads();
    if (slice != 0) return;
    const int rs = a.rpt_shift;
    const int nout = gcount << rs;
    for (int idx0 = 0; idx0 < nout; idx0 += 64) {
        const int idx = idx0 + lane;
        const bool valid = idx < nout;
        const int idc = valid ? idx : 0;
        const int gl = idc >> rs, rr = idc & (a.rpt - 1);
        const int row = ((gbase + gl) << rs) + rr;
        const int2 *src = abuf + (((gl * m) << rs) + rr);
        double z = 0.0;
        for (int i0 = 0; i0 < m; i0 += 4) {
            // four layers at a time: the LDS reads are issued together, the arithmetic follows
            int2 v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = (i0 + k < m) ? i0 + k : m - 1;
                v[k] = src[i << rs];
                for (int sl = 1; sl < a.csplit; ++sl) {
                    const int2 w = src[(size_t)sl * a.abuf_words + (i << rs)];
                    v[k].x += w.x;
                    v[k].y += w.y;
                }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = i0 + k;
                if (i < m) {
                    if (a.A) {
                        if (valid && row < a.R)
                            a.A[((size_t)i * a.batch + n) * (size_t)a.R + row] =
                                (long long)v[k].x + ((long long)v[k].y << 16);
                    } else {
                        const float si =
                            __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(scv), i));
                        z += (double)si * ((double)v[k].x + (double)v[k].y * 65536.0);
                    }
                }
            }
        }
        if (!a.A && valid && row < a.R) a.Y[(size_t)n * a.R + row] = (float)(z * a.out_scale);
    }
}

static int ilog2(int v)
{
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

int launch_matvec(const uint32_t *packed, const float *scales, const Layout &L, int bits_used, int frac_bits,
                  const uint32_t *planes, const int *meta, int batch, float *Y, long long *A, hipStream_t st)
{
    MatvecArgs a;
    a.packed = packed; a.planes = planes; a.meta = meta; a.scales = scales; a.Y = Y; a.A = A;
    a.layer_words = L.layer_words;
    a.packed_bytes = packed_bytes(L);
    a.R = L.rows; a.cwp = L.cwp; a.ws = L.ws; a.rpt = L.rpt; a.csplit = L.csplit;
    a.ws_shift = ilog2(L.ws);
    a.rpt_shift = ilog2(L.rpt);
    a.csplit_magic = 65536 / L.csplit + 1;   // (wave * magic) >> 16 == wave / csplit for wave < 8
    a.rwaves = L.csplit == 1 ? 4 : (L.csplit <= 4 ? 2 : 1);
    if (a.csplit * a.rwaves > kMaxWavesPerWG) a.rwaves = 1;
    a.m = bits_used;
    a.num_rowgroups = L.rows_p / L.rpt;
    a.batch = batch;
    a.out_scale = ldexp(1.0, -frac_bits);
    // Waves: one per SIMD (1024) while a wave then has at most 8 tiles, else two per SIMD; every wave repeats the
    // plane fetch and the epilogue, so more waves only pay off once each has enough tiles to overlap with.
    const long long tiles_per_wave_at_1024 = (long long)a.num_rowgroups * bits_used * a.csplit / 1024;
    const int waves_total = tiles_per_wave_at_1024 <= 8 ? 1024 : 2048;
    int target_wgs = waves_total / (a.csplit * a.rwaves);
    if (target_wgs < 1) target_wgs = 1;
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
    size_t smem = (size_t)waves * kRedTiles * 64 * sizeof(int2) + (size_t)waves * a.abuf_words * sizeof(int2);
    if (smem > 64 * 1024) {
        // more than the default 64 KB of dynamic LDS (a CU of this GPU has 160 KB)
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_matvec),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL(k_matvec, dim3((unsigned)nwg, (unsigned)batch), dim3(waves * 64), smem, st, a);
    return (int)hipGetLastError();
}

}  // namespace pb
