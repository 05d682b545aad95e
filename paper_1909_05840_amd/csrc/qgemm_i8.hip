// Forward of the group-quantized linear layer on the gfx950 int8 matrix cores.
//
//   acc[t,n] = sum_j x'[t,j] * b[n,j]       v_mfma_i32_32x32x32_i8, int32 accumulators
//   A4[t,n]  = 4*acc + 2*e*rs_x[t] + 2*rs_w[n] + K
//   Y[t,n]   = (h_x*h_g(n)) * float(A4) (+ bias[n])
//
// b is the int8 the matrix core sees: the unsigned code u itself for 2/3/4 bits (e = -L) and
// u - 128 for 8 bits (e = +1); either way A4 equals sum_j (2x'+1)(2u-L), the integer that the
// integer product of the codes, de-quantized once afterwards (App., last paragraph), has to produce.
//
// Three kernels, chosen by shape (launch_bits):
//   qgemm_i8_kernel     register-staged: the token tile goes global -> registers -> LDS, the packed weights never
//                       touch LDS (the packed layout stores, per 32-neuron block and 64-feature unit, one slot per
//                       lane, so a wavefront fetches its B operand with one coalesced load).  Small tiles for
//                       problems of few tiles, and any K that is a multiple of 64.
//   qgemm_i8_dma_kernel both operands copied global -> LDS by the load unit itself (global_load_lds_dwordx4, no
//                       registers involved) through a ring of stages; every wavefront copies and multiplies; two
//                       workgroups per CU.
//   qgemm_i8_ws_kernel  the same data path with the work split by role (copy wavefronts / MFMA wavefronts), a
//                       persistent grid that walks the tiles of one or several problems (a table of problems is the
//                       kernel argument), epilogue parameters staged in LDS; optionally with the copy wavefronts on
//                       a SIMD of their own (128x96 tiles; two workgroups per CU when there are more tiles than CUs:
//                       one's write-out runs under the other's K-loop), an 8-bit output, per-token scales,
//                       asymmetric group ranges.
// In all of them the token tile sits in LDS as dense 128-byte rows whose 16-byte chunks are XOR-swizzled by the
// row number, so that the MFMA fragment reads are free of bank conflicts, and the k-bit codes are expanded to
// int8 with a few byte-parallel shifts and masks in registers, right in front of the MFMA that consumes them.
// Workgroups are renumbered so that the ones sharing a token panel run on the same XCD (same L2).
#include "qb_common.hpp"

namespace qb {
namespace {

// a*b + c for |a|, |b| < 2^23 (full-rate 24-bit multiplier instead of the quarter-rate 32-bit one)
__device__ __forceinline__ int qb_mad24(int a, int b, int c) { return __mul24(a, b) + c; }

// A4 = 4*acc + corr.  The result fits int32 for every K the library accepts, but 4*acc alone can reach 2^31 at
// K = 32768 with end-of-range operands: the sum is formed modulo 2^32 in unsigned arithmetic.
__device__ __forceinline__ int qb_a4(int acc, int corr) { return (int)(4u * (uint32_t)acc + (uint32_t)corr); }

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// Asymmetric group ranges (weights Delta*u + q0, u = 0..L): with R = sum_j (2x'+1) = 2*rs_x + K and
// S = sum_j (2x'+1)*u = (A4 + L*R)/2 the output is h_x*(Delta*S + q0*R).  A4 and R are even (K is), and
// S = A4/2 + L*(R/2) stays inside int32 for every K the library accepts.  rh = R/2 = rs_x + K/2.
__device__ __forceinline__ float asym_value(int a4, int rh, int L, float hx, float delta, float q0)
{
    const int S = (a4 >> 1) + L * rh;
    return hx * (delta * (float)S + q0 * (float)(2 * rh));
}

// bid: the workgroup's number among the tiles_m * tiles_n workgroups of this problem
template <int BITS, int TM, int TN, int WM, int WN, int KU>
__device__ __forceinline__ void qgemm_i8_body(
    const int8_t *__restrict__ Xq, const int32_t *__restrict__ rs_x, const uint8_t *__restrict__ packed,
    const float *__restrict__ h, const int32_t *__restrict__ rs_w, const float *__restrict__ bias,
    float *__restrict__ Y, int32_t *__restrict__ A4out, int T, int N, int K, int rows_per_group, float hx,
    int tiles_m, int tiles_n, const float *__restrict__ hx_rows, const float *__restrict__ q0, const int bid)
{
    // hx_rows: one activation scale per token (dynamic range) instead of hx, or null
    // q0: asymmetric group ranges: h holds Delta and q0 the lower end of every group, or null
    constexpr int THREADS = 64 * WM * WN;
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 64 * KU, LDA = BK + 16;
    constexpr int CHUNKS_PER_ROW = BK / 16;
    constexpr int A_PER_THREAD = BM * CHUNKS_PER_ROW / THREADS;
    static_assert(BM * CHUNKS_PER_ROW % THREADS == 0, "A tile must split evenly over the threads");
    constexpr int SLOT = 4 * BITS;  // bytes per slot

    __shared__ __align__(16) uint8_t lds[2][BM * LDA];

    // ---- which tile: blocks are dealt round-robin to the 8 XCDs; give each XCD a contiguous
    // range of tiles (n fastest) so that a token panel is fetched into one L2 only
    const int nwg = tiles_m * tiles_n;
    int logical;
    {
        const int xcd = bid & 7, idx = bid >> 3;
        const int q = nwg >> 3, r = nwg & 7;
        logical = xcd * q + (xcd < r ? xcd : r) + idx;
    }
    const int tile_m = logical / tiles_n, tile_n = logical - tile_m * tiles_n;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave - wm * WN;
    const int l32 = lane & 31, hf = lane >> 5;

    // ---- global sources
    const int8_t *a_src[A_PER_THREAD];
    int a_dst[A_PER_THREAD];
#pragma unroll
    for (int i = 0; i < A_PER_THREAD; ++i) {
        const int c = tid + i * THREADS;
        const int row = c / CHUNKS_PER_ROW, kc = c - row * CHUNKS_PER_ROW;
        int t = tile_m * BM + row;
        t = t < T ? t : T - 1;  // rows past the end re-read the last row; their outputs are masked
        a_src[i] = Xq + (size_t)t * K + kc * 16;
        a_dst[i] = row * LDA + kc * 16;
    }
    const int kunits = K >> 6;
    const int ncb = (N + 31) >> 5;
    const uint8_t *b_src[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        int cb = tile_n * (BN / 32) + wn * TN + tn;
        cb = cb < ncb ? cb : ncb - 1;
        b_src[tn] = packed + ((size_t)cb * kunits * 64 + lane) * SLOT;
    }

    v16i acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0;

    v4u areg[A_PER_THREAD];
    uint32_t bnext[TN][KU][BITS], bcur[TN][KU][BITS];
    const int a_frag_base = (wm * TM * 32 + l32) * LDA + hf * 32;

// global -> registers for K-step `step`: the token tile (to be staged in LDS) and this lane's slots
#define QB_LOAD_GLOBAL(step, BDST)                                                                        \
    {                                                                                                     \
        _Pragma("unroll") for (int i = 0; i < A_PER_THREAD; ++i)                                          \
            areg[i] = *reinterpret_cast<const v4u *>(a_src[i] + (size_t)(step) * BK);                    \
        _Pragma("unroll") for (int tn = 0; tn < TN; ++tn)                                                 \
            _Pragma("unroll") for (int kk = 0; kk < KU; ++kk) {                                           \
                const uint32_t *p_ =                                                                      \
                    reinterpret_cast<const uint32_t *>(b_src[tn] + (size_t)((step) * KU + kk) * 64 * SLOT); \
                _Pragma("unroll") for (int i = 0; i < BITS; ++i) BDST[tn][kk][i] = p_[i];                 \
            }                                                                                             \
    }
#define QB_STORE_LDS(buf)                                                                                 \
    {                                                                                                     \
        _Pragma("unroll") for (int i = 0; i < A_PER_THREAD; ++i)                                          \
            *reinterpret_cast<v4u *>(&lds[buf][a_dst[i]]) = areg[i];                                      \
    }
// all MFMAs of one K-step: expand this lane's codes to int8 in registers, A fragments from LDS
#define QB_COMPUTE(buf)                                                                                   \
    {                                                                                                     \
        const uint8_t *abuf = lds[buf];                                                                   \
        _Pragma("unroll") for (int kk = 0; kk < KU; ++kk) {                                               \
            uint32_t d[TN][8];                                                                            \
            _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) {                                           \
                unpack_run<BITS>(bcur[tn][kk], d[tn]);                                                    \
                if constexpr (BITS == 8) {                                                                \
                    _Pragma("unroll") for (int i = 0; i < 8; ++i) d[tn][i] ^= 0x80808080u;                \
                }                                                                                         \
            }                                                                                             \
            _Pragma("unroll") for (int sub = 0; sub < 2; ++sub) {                                         \
                v4i a[TM], b[TN];                                                                         \
                _Pragma("unroll") for (int tm = 0; tm < TM; ++tm) a[tm] = *reinterpret_cast<const v4i *>( \
                    abuf + a_frag_base + tm * 32 * LDA + kk * 64 + sub * 16);                             \
                _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) {                                       \
                    b[tn][0] = (int)d[tn][4 * sub + 0];                                                   \
                    b[tn][1] = (int)d[tn][4 * sub + 1];                                                   \
                    b[tn][2] = (int)d[tn][4 * sub + 2];                                                   \
                    b[tn][3] = (int)d[tn][4 * sub + 3];                                                   \
                }                                                                                         \
                _Pragma("unroll") for (int tm = 0; tm < TM; ++tm)                                         \
                    _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) acc[tm][tn] =                       \
                        __builtin_amdgcn_mfma_i32_32x32x32_i8(a[tm], b[tn], acc[tm][tn], 0, 0, 0);        \
            }                                                                                             \
        }                                                                                                 \
    }
#define QB_ROTATE_B()                                                                                     \
    {                                                                                                     \
        _Pragma("unroll") for (int tn = 0; tn < TN; ++tn)                                                 \
            _Pragma("unroll") for (int kk = 0; kk < KU; ++kk)                                             \
                _Pragma("unroll") for (int i = 0; i < BITS; ++i) bcur[tn][kk][i] = bnext[tn][kk][i];      \
    }

    const int nsteps = K / BK;
    QB_LOAD_GLOBAL(0, bcur)
    QB_STORE_LDS(0)
    __syncthreads();
    // steady state: fetch step s+1 while the matrix cores work on step s (no branches inside)
    for (int s = 0; s < nsteps - 1; ++s) {
        QB_LOAD_GLOBAL(s + 1, bnext)
        __builtin_amdgcn_sched_barrier(0);  // keep the fetches ahead of the MFMAs: their latency hides under them
        QB_COMPUTE(s & 1)
        __builtin_amdgcn_sched_barrier(0);
        QB_STORE_LDS((s + 1) & 1)
        QB_ROTATE_B()
        __syncthreads();
    }
    QB_COMPUTE((nsteps - 1) & 1)
#undef QB_LOAD_GLOBAL
#undef QB_STORE_LDS
#undef QB_COMPUTE
#undef QB_ROTATE_B

    // ---- epilogue: exact integer corrections, then one scale per column
    constexpr int L = (1 << BITS) - 1;
    constexpr int E2 = (BITS == 8) ? 2 : -2 * L;  // 2*e
    const bool interior = (tile_m + 1) * BM <= T && (tile_n + 1) * BN <= N;  // uniform over the workgroup
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int n = tile_n * BN + (wn * TN + tn) * 32 + l32;
        const bool n_ok = n < N;
        const int nn = n_ok ? n : N - 1;
        const int coln = 2 * rs_w[nn] + K;
        const float hg = h[nn / rows_per_group];
        const float scale = hx * hg;
        const float bv = bias ? bias[nn] : 0.0f;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int t0 = tile_m * BM + (wm * TM + tm) * 32 + 4 * hf;
            if (q0) {
                const float zn = q0[nn / rows_per_group];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = t0 + 8 * (i >> 2) + (i & 3);
                    if (t < T && n_ok) {
                        const int a4 = qb_a4(acc[tm][tn][i], E2 * rs_x[t] + coln);
                        const size_t at = (size_t)t * N + n;
                        Y[at] = asym_value(a4, rs_x[t] + (K >> 1), L, hx_rows ? hx_rows[t] : hx, hg, zn) + bv;
                        if (A4out) A4out[at] = a4;
                    }
                }
            } else if (hx_rows) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = t0 + 8 * (i >> 2) + (i & 3);
                    if (t < T && n_ok) {
                        const int a4 = qb_a4(acc[tm][tn][i], E2 * rs_x[t] + coln);
                        const size_t at = (size_t)t * N + n;
                        Y[at] = (hx_rows[t] * hg) * (float)a4 + bv;
                        if (A4out) A4out[at] = a4;
                    }
                }
            } else if (interior) {
                int rx[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) rx[i] = rs_x[t0 + 8 * (i >> 2) + (i & 3)];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = t0 + 8 * (i >> 2) + (i & 3);
                    const int a4 = qb_a4(acc[tm][tn][i], qb_mad24(E2, rx[i], coln));
                    const size_t at = (size_t)t * N + n;
                    Y[at] = scale * (float)a4 + bv;
                    if (A4out) A4out[at] = a4;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = t0 + 8 * (i >> 2) + (i & 3);
                    if (t < T && n_ok) {
                        const int a4 = qb_a4(acc[tm][tn][i], E2 * rs_x[t] + coln);
                        const size_t at = (size_t)t * N + n;
                        Y[at] = scale * (float)a4 + bv;
                        if (A4out) A4out[at] = a4;
                    }
                }
            }
        }
    }
}

template <int BITS, int TM, int TN, int WM, int WN, int KU>
__global__ __launch_bounds__(64 * WM * WN) void qgemm_i8_kernel(
    const int8_t *__restrict__ Xq, const int32_t *__restrict__ rs_x, const uint8_t *__restrict__ packed,
    const float *__restrict__ h, const int32_t *__restrict__ rs_w, const float *__restrict__ bias,
    float *__restrict__ Y, int32_t *__restrict__ A4out, int T, int N, int K, int rows_per_group, float hx,
    int tiles_m, int tiles_n, const float *__restrict__ hx_rows, const float *__restrict__ q0)
{
    qgemm_i8_body<BITS, TM, TN, WM, WN, KU>(Xq, rs_x, packed, h, rs_w, bias, Y, A4out, T, N, K, rows_per_group, hx, tiles_m,
                                            tiles_n, hx_rows, q0, blockIdx.x);
}

// Several few-tile problems (small token counts: the inference regime, where a launch costs more than its work) in one
// launch of the 32x64-tile form: workgroup w serves tile w - first_wg[j] of problem j; a problem's workgroups start at
// a multiple of 8, so that its tiles keep their XCD (the fill-up workgroups leave at once).
struct SmallProblem {
    const int8_t *Xq;
    const int32_t *rs_x;
    const uint8_t *packed;
    const float *h;
    const int32_t *rs_w;
    const float *bias;
    float *Y;
    int T, N, K, rows_per_group;
    float hx;
    int tiles_m, tiles_n;
};
struct SmallGroup {
    int n;
    int first_wg[QB_MAX_BATCH + 1];
    SmallProblem p[QB_MAX_BATCH];
};
template <int BITS, int KU>
__global__ __launch_bounds__(128) void qgemm_i8_small_group_kernel(const SmallGroup g)
{
    int j = 0;
    while (j + 1 < g.n && (int)blockIdx.x >= g.first_wg[j + 1]) ++j;
    const SmallProblem &p = g.p[j];
    const int local = blockIdx.x - g.first_wg[j];
    if (local >= p.tiles_m * p.tiles_n) return;  // (uniform over the workgroup)
    qgemm_i8_body<BITS, 1, 1, 1, 2, KU>(p.Xq, p.rs_x, p.packed, p.h, p.rs_w, p.bias, p.Y, nullptr, p.T, p.N, p.K,
                                        p.rows_per_group, p.hx, p.tiles_m, p.tiles_n, nullptr, nullptr, local);
}

// global -> LDS copy by the load unit: the global address of a lane is a wavefront-uniform base (in SGPRs) plus
// the lane's 32-bit byte offset, the data of lane l lands at LDS address m0 + 16*l (also for the 12-byte form).
// Written as inline assembly on purpose: the compiler then keeps no book on these copies, and the kernel states
// itself, with wait_vmcnt, which of them must have landed before a barrier.
__device__ __forceinline__ void copy16_to_lds(const void *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0" ::"s"(base), "v"(off), "s"(lds_addr) : "memory", "m0");
}
__device__ __forceinline__ void copy12_to_lds(const void *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx3 %1, %0" ::"s"(base), "v"(off), "s"(lds_addr) : "memory", "m0");
}

template <int BITS> struct SlotRead;  // one lane's slot (32 codes) out of LDS
template <> struct SlotRead<2> {
    static __device__ __forceinline__ void get(const uint8_t *p, uint32_t (&o)[2])
    {
        const uint2 v = *reinterpret_cast<const uint2 *>(p);
        o[0] = v.x; o[1] = v.y;
    }
};
template <> struct SlotRead<3> {
    typedef unsigned int v3u __attribute__((ext_vector_type(3)));
    static __device__ __forceinline__ void get(const uint8_t *p, uint32_t (&o)[3])
    {
        const v3u v = *reinterpret_cast<const v3u *>(p);
        o[0] = v[0]; o[1] = v[1]; o[2] = v[2];
    }
};
template <> struct SlotRead<4> {
    static __device__ __forceinline__ void get(const uint8_t *p, uint32_t (&o)[4])
    {
        const v4u v = *reinterpret_cast<const v4u *>(p);
        o[0] = v[0]; o[1] = v[1]; o[2] = v[2]; o[3] = v[3];
    }
};
template <> struct SlotRead<8> {
    static __device__ __forceinline__ void get(const uint8_t *p, uint32_t (&o)[8])
    {
        const v4u a = *reinterpret_cast<const v4u *>(p), b = *reinterpret_cast<const v4u *>(p + 16);
        o[0] = a[0]; o[1] = a[1]; o[2] = a[2]; o[3] = a[3];
        o[4] = b[0]; o[5] = b[1]; o[6] = b[2]; o[7] = b[3];
    }
};

// vmcnt(N) with the other counters left alone (gfx9 encoding of s_waitcnt's immediate)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0070 | 0x0F00);
}

// Main kernel, K a multiple of 128.  One K-step is 128 features = two 64-code units.
// Both operands are copied global -> LDS by the load unit (no staging registers):
//   tokens : dense rows of 128 bytes, 16-byte chunks XOR-swizzled with the row number
//   weights: the packed slots as they are, [32-neuron block][unit][lane][slot]; a wavefront
//            then reads one slot per lane (conflict free) and expands it in registers
// The copies run NSTAGE-1 steps ahead of the matrix cores through a ring of NSTAGE stage
// buffers; a step ends with "the copies for the next step have landed" (vmcnt leaves the younger
// ones in flight; copies return in issue order) and a workgroup barrier.
template <int BITS, int TM, int TN, int WM, int WN, int NSTAGE>
__global__ __launch_bounds__(64 * WM * WN) void qgemm_i8_dma_kernel(
    const int8_t *__restrict__ Xq, const int32_t *__restrict__ rs_x, const uint8_t *__restrict__ packed,
    const float *__restrict__ h, const int32_t *__restrict__ rs_w, const float *__restrict__ bias,
    float *__restrict__ Y, int32_t *__restrict__ A4out, int T, int N, int K, int rows_per_group, float hx,
    int tiles_m, int tiles_n)
{
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "ring of 2..4 stages");
    constexpr int NW = WM * WN;
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 128;
    constexpr int A_DMA = BM / 8 / NW;          // per wavefront and step; each fills 8 rows of 128 bytes
    static_assert(BM % (8 * NW) == 0, "token tile must split into 8-row blocks per wavefront");
    constexpr int SLOT = 4 * BITS;               // bytes per slot in memory
    constexpr int CH = (BITS == 3) ? 12 : 16;    // bytes one lane moves per weight copy instruction
    constexpr int LSLOT = (BITS == 3) ? 16 : SLOT;  // bytes per slot in LDS: a 12-byte copy lands at a 16-byte stride
    constexpr int PAIR = 128 * SLOT;             // bytes of one 32-neuron block x two units (contiguous in memory)
    constexpr int LPAIR = 128 * LSLOT;           // the same block in LDS
    constexpr int PARTS = PAIR / (64 * CH);      // copy instructions per pair; each fills 1024 bytes of LDS
    constexpr int B_TOTAL = (BN / 32) * PARTS;   // copy instructions per step for the whole workgroup
    constexpr int B_DMA = (B_TOTAL + NW - 1) / NW;
    constexpr int PER = A_DMA + B_DMA;           // copy instructions per wavefront and step
    constexpr int D = NSTAGE - 1;                // how many steps the copies run ahead
    constexpr int A_BYTES = BM * BK, B_BYTES = (BN / 32) * LPAIR;

    constexpr int STAGE_BYTES = A_BYTES + B_BYTES;  // tokens first, then weights
    __shared__ __align__(1024) uint8_t lds[NSTAGE * STAGE_BYTES];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave - wm * WN;
    const int l32 = lane & 31, hf = lane >> 5;

    // Workgroups are persistent: each walks over tiles work = blockIdx.x, + gridDim.x, ... (the
    // grid is a multiple of 8, so a workgroup stays on the tiles of its own XCD's range).
    const int nwg = tiles_m * tiles_n;
    for (int work = blockIdx.x; work < nwg; work += gridDim.x) {
    int logical;
    {
        const int xcd = work & 7, idx = work >> 3;
        const int q = nwg >> 3, r = nwg & 7;
        logical = xcd * q + (xcd < r ? xcd : r) + idx;
    }
    const int tile_m = logical / tiles_n, tile_n = logical - tile_m * tiles_n;

    // ---- token tile copies: lane l of an instruction fills physical chunk l%8 of row l/8 of an
    // 8-row block, which holds logical chunk (l%8) ^ (row%8)
    const int8_t *a_base = Xq + (size_t)tile_m * BM * K;
    const int last_row = T - 1 - tile_m * BM;  // rows past the end re-read the last one; outputs masked
    uint32_t a_off[A_DMA];
#pragma unroll
    for (int i = 0; i < A_DMA; ++i) {
        int row = (i * NW + wave) * 8 + (lane >> 3);
        row = row < last_row ? row : last_row;
        a_off[i] = (uint32_t)row * (uint32_t)K + (uint32_t)(((lane & 7) ^ (lane >> 3)) * 16);
    }
    // ---- weight copies: instruction j moves part j%PARTS of the pair of block j/PARTS.  Every
    // wavefront issues the same number of copies (the vmcnt arithmetic relies on it): surplus
    // ones repeat an earlier copy, writing the same bytes to the same place.
    const int kunits = K >> 6;
    const int ncb = (N + 31) >> 5;
    // (addresses: a wavefront-uniform base per tile and step, a 32-bit byte offset per lane and copy)
    const int cb0 = tile_n * (BN / 32);
    const uint8_t *b_base = packed + (size_t)cb0 * kunits * 64 * SLOT;
    uint32_t b_off[B_DMA];
    int b_ldst[B_DMA];
#pragma unroll
    for (int i = 0; i < B_DMA; ++i) {
        const int j = (i * NW + wave) % B_TOTAL;
        const int pair = j / PARTS, part = j - pair * PARTS;
        int cb = cb0 + pair;
        cb = cb < ncb ? cb : ncb - 1;  // blocks past the end re-read the last one; outputs masked
        b_off[i] = (uint32_t)(cb - cb0) * (uint32_t)(kunits * 64 * SLOT) + part * 64 * CH + lane * CH;
        b_ldst[i] = pair * LPAIR + part * 1024;
    }
    // ---- fragment reads.  tokens: row = wm*TM*32 + tm*32 + l32, logical chunk = kk*4 + hf*2 + sub
    const int p0 = (hf * 2) ^ (l32 & 7);
    const int frag_row = (wm * TM * 32 + l32) * BK;
    int a_frag[4];
    a_frag[0] = frag_row + ((p0 ^ 0) << 4);  // kk 0, sub 0
    a_frag[1] = frag_row + ((p0 ^ 1) << 4);  // kk 0, sub 1
    a_frag[2] = frag_row + ((p0 ^ 4) << 4);  // kk 1, sub 0
    a_frag[3] = frag_row + ((p0 ^ 5) << 4);  // kk 1, sub 1
    const int b_frag = wn * TN * LPAIR + lane * LSLOT;  // + tn*LPAIR + kk*64*LSLOT

    v16i acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0;

#define QB_FETCH(step, stage)                                                                             \
    {                                                                                                     \
        const uint32_t st_ = lds_base + (stage) * STAGE_BYTES;                                            \
        _Pragma("unroll") for (int i = 0; i < B_DMA; ++i) {                                               \
            if constexpr (BITS == 3) copy12_to_lds(b_base + (size_t)(step) * PAIR, b_off[i], st_ + A_BYTES + b_ldst[i]); \
            else copy16_to_lds(b_base + (size_t)(step) * PAIR, b_off[i], st_ + A_BYTES + b_ldst[i]);      \
        }                                                                                                 \
        _Pragma("unroll") for (int i = 0; i < A_DMA; ++i)                                                 \
            copy16_to_lds(a_base + (size_t)(step) * BK, a_off[i], st_ + (i * NW + wave) * 1024);          \
    }
#define QB_MMA(stage)                                                                                     \
    {                                                                                                     \
        const uint8_t *lds_a = lds + (stage) * STAGE_BYTES, *lds_b = lds_a + A_BYTES;                     \
        _Pragma("unroll") for (int kk = 0; kk < 2; ++kk) {                                                \
            uint32_t d[TN][8];                                                                            \
            _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) {                                           \
                uint32_t raw[BITS];                                                                       \
                SlotRead<BITS>::get(lds_b + b_frag + tn * LPAIR + kk * 64 * LSLOT, raw);                  \
                unpack_run<BITS>(raw, d[tn]);                                                             \
                if constexpr (BITS == 8) {                                                                \
                    _Pragma("unroll") for (int i = 0; i < 8; ++i) d[tn][i] ^= 0x80808080u;                \
                }                                                                                         \
            }                                                                                             \
            _Pragma("unroll") for (int sub = 0; sub < 2; ++sub) {                                         \
                v4i a[TM], b[TN];                                                                         \
                _Pragma("unroll") for (int tm = 0; tm < TM; ++tm)                                         \
                    a[tm] = *reinterpret_cast<const v4i *>(lds_a + a_frag[kk * 2 + sub] + tm * 32 * BK);  \
                _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) {                                       \
                    b[tn][0] = (int)d[tn][4 * sub + 0];                                                   \
                    b[tn][1] = (int)d[tn][4 * sub + 1];                                                   \
                    b[tn][2] = (int)d[tn][4 * sub + 2];                                                   \
                    b[tn][3] = (int)d[tn][4 * sub + 3];                                                   \
                }                                                                                         \
                _Pragma("unroll") for (int tm = 0; tm < TM; ++tm)                                         \
                    _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) acc[tm][tn] =                       \
                        __builtin_amdgcn_mfma_i32_32x32x32_i8(a[tm], b[tn], acc[tm][tn], 0, 0, 0);        \
            }                                                                                             \
        }                                                                                                 \
    }

// End of a step.  A bare s_barrier, not __syncthreads(): the fence inside the latter would wait
// for every copy in flight (vmcnt 0) and with that undo the run-ahead.  What the barrier has to
// order: this wavefront's copies for the next step have landed (wait_vmcnt), and its LDS reads of the
// step have returned: the stage is overwritten by copies that start right behind the barrier.  The
// second needs the explicit wait for the LDS counter: the compiler is free to let the MFMAs that
// consume the step's last fragments follow below the barrier, and the reads would then still be
// queued in the LDS when the wavefront arrives (seen as wrong results in the backward's kernel, which
// has the same structure, when another stream's kernel kept the CU's LDS busy).
// The empty asm keeps the compiler from moving LDS reads of the next step above the barrier.
#define QB_STEP_BARRIER()                                                                                 \
    {                                                                                                     \
        __builtin_amdgcn_s_waitcnt(0xC07F); /* lgkmcnt(0) */                                              \
        __builtin_amdgcn_s_barrier();                                                                     \
        asm volatile("" ::: "memory");                                                                    \
    }

    const int nsteps = K / BK;
    // prologue: start the copies of the first D steps, wait for step 0 only
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < nsteps) QB_FETCH(u, u)
    if (nsteps >= D) wait_vmcnt<(D - 1) * PER>();
    else wait_vmcnt<0>();
    QB_STEP_BARRIER();

    int s = 0;
    for (; s + NSTAGE <= nsteps; s += NSTAGE) {
#pragma unroll
        for (int u = 0; u < NSTAGE; ++u) {
            const bool more = s + u + D < nsteps;  // uniform
            if (more) QB_FETCH(s + u + D, (u + D) % NSTAGE)
            QB_MMA(u)
            if (more) wait_vmcnt<(D - 1) * PER>();  // copies for the next step have landed, younger ones fly on
            else wait_vmcnt<0>();
            QB_STEP_BARRIER();
        }
    }
    // tail: fewer than NSTAGE steps left, all their copies are already issued
#pragma unroll
    for (int u = 0; u < NSTAGE - 1; ++u)
        if (s + u < nsteps) {
            QB_MMA(u)
            wait_vmcnt<0>();
            QB_STEP_BARRIER();
        }
#undef QB_FETCH
#undef QB_MMA
#undef QB_STEP_BARRIER

    // ---- epilogue: exact integer corrections, then one scale per column.  Everything the
    // stores depend on is loaded first: a load issued between two stores would make the wavefront
    // wait for the older store to complete (loads and stores share one in-order counter) and turn
    // the write-out into a chain of round trips.
    constexpr int L = (1 << BITS) - 1;
    constexpr int E2 = (BITS == 8) ? 2 : -2 * L;  // 2*e
    const bool interior = (tile_m + 1) * BM <= T && (tile_n + 1) * BN <= N;  // uniform over the workgroup
    int coln[TN];
    float scale[TN], bv[TN];
    bool n_ok[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int n = tile_n * BN + (wn * TN + tn) * 32 + l32;
        n_ok[tn] = n < N;
        const int nn = n_ok[tn] ? n : N - 1;
        coln[tn] = 2 * rs_w[nn] + K;
        scale[tn] = hx * h[nn / rows_per_group];
        bv[tn] = bias ? bias[nn] : 0.0f;
    }
    if (interior && A4out == nullptr) {
        // fast path (uniform branch): straight-line code, one scalar base per 32x32 block and one
        // 32-bit lane offset per accumulator register
        const int t_wave = tile_m * BM + wm * TM * 32, n_wave = tile_n * BN + wn * TN * 32;
        float *y_wave = Y + (size_t)t_wave * N + n_wave;
        const int32_t *rx_wave = rs_x + t_wave;
        uint32_t voff[16];
#pragma unroll
        for (int i = 0; i < 16; ++i)
            voff[i] = ((uint32_t)(4 * hf + 8 * (i >> 2) + (i & 3)) * (uint32_t)N + (uint32_t)l32) * 4u;
        int rx[TM][16];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int i = 0; i < 16; ++i) rx[tm][i] = rx_wave[tm * 32 + 4 * hf + 8 * (i >> 2) + (i & 3)];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                char *y_blk = reinterpret_cast<char *>(y_wave + (size_t)tm * 32 * N + tn * 32);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int a4 = qb_a4(acc[tm][tn][i], qb_mad24(E2, rx[tm][i], coln[tn]));
                    __builtin_nontemporal_store(scale[tn] * (float)a4 + bv[tn], reinterpret_cast<float *>(y_blk + voff[i]));
                }
            }
    } else {
        // edge tiles and the debug output: every element checked
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int t0 = tile_m * BM + (wm * TM + tm) * 32 + 4 * hf;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int n = tile_n * BN + (wn * TN + tn) * 32 + l32;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = t0 + 8 * (i >> 2) + (i & 3);
                    if (t < T && n_ok[tn]) {
                        const int a4 = qb_a4(acc[tm][tn][i], E2 * rs_x[t] + coln[tn]);
                        const size_t at = (size_t)t * N + n;
                        Y[at] = scale[tn] * (float)a4 + bv[tn];
                        if (A4out) A4out[at] = a4;
                    }
                }
            }
        }
    }
    }  // persistent tile loop
}

// 4-byte form of the global -> LDS copy: lane l's dword lands at m0 + 4*l
__device__ __forceinline__ void copy4_to_lds(const void *g, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(g), "s"(lds_addr) : "memory", "m0");
}

// Epilogue of the role-split kernel.  Its per-token and per-neuron parameters do not come from global
// memory but from a block in LDS that a producer wavefront filled for the tile (BM ints rs_x, then BN
// each of rs_w, h of the neuron's group, bias, then BM per-token scales and, with asymmetric ranges, BN values of q0 of
// the neuron's group; indices past the end of the matrix were clamped).  The
// consumer wavefronts thus issue no global loads at all: their memory counter holds stores only and is
// never waited on, so the stores of one tile need not have completed before the next tile's go out.
// acc[tm][tn][r]: token tl + 32*tm + 8*(r/4) + (r%4) of the tile (tl contains 4*hf), neuron nl + 32*tn
// (nl contains l32).  A4 = 4*acc + 2e*rs_x[t] + 2*rs_w[n] + K,  Y = (h_x*h_g(n)) * float(A4) + bias[n];
// dyn: h_x per token; asym_L = 2^k - 1: asymmetric group ranges, Y = asym_value(...) + bias[n].
template <int BM, int BN>
__device__ __forceinline__ void store_block_lds(const v16i &acc, const uint8_t *pp, int e2, int tl, int nl, int t0, int n0,
                                                int T, int N, int K, float hx, bool has_bias, bool fast,
                                                float *__restrict__ Y, int32_t *__restrict__ A4out, bool dyn = false,
                                                int asym_L = 0)
{
    // one 32x32 block: acc[r] is token tl + 8*(r/4) + (r%4) of the tile, neuron nl
    const int *p_rx = reinterpret_cast<const int *>(pp);
    const int *p_rw = p_rx + BM;
    const float *p_h = reinterpret_cast<const float *>(p_rw + BN), *p_b = p_h + BN;
    const int coln = 2 * p_rw[nl] + K;
    const float scale = hx * p_h[nl];
    const float bv = has_bias ? p_b[nl] : 0.0f;
    // per row: the scale.  dyn: one activation scale per token, the tile's BM of them follow the bias in the
    // parameter block; otherwise the one scale of the call.
    float sc[16];
    if (dyn) {
        const float *p_hx = p_b + BN;
        const float hg = p_h[nl];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v = *reinterpret_cast<const float4 *>(p_hx + tl + 8 * q);
            sc[4 * q + 0] = v.x * hg;
            sc[4 * q + 1] = v.y * hg;
            sc[4 * q + 2] = v.z * hg;
            sc[4 * q + 3] = v.w * hg;
        }
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[r] = scale;
    }
    int rx[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int4 v = *reinterpret_cast<const int4 *>(p_rx + tl + 8 * q);
        rx[4 * q + 0] = qb_mad24(e2, v.x, coln);  // |rs_x| <= 128*K < 2^23: the 24-bit multiply is exact and full rate
        rx[4 * q + 1] = qb_mad24(e2, v.y, coln);
        rx[4 * q + 2] = qb_mad24(e2, v.z, coln);
        rx[4 * q + 3] = qb_mad24(e2, v.w, coln);
    }
    if (asym_L) {  // asymmetric group ranges: Delta in the place of h, q0 behind the per-token scales
        const float dn = p_h[nl], zn = (p_b + BN + BM)[nl];
        float hr[16];  // the activation scale of every row: the call's, or the token's own
        if (dyn) {
            const float *p_hx = p_b + BN;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = *reinterpret_cast<const float4 *>(p_hx + tl + 8 * q);
                hr[4 * q + 0] = v.x; hr[4 * q + 1] = v.y; hr[4 * q + 2] = v.z; hr[4 * q + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) hr[r] = hx;
        }
        int rh[16];  // R/2 = rs_x + K/2 per row
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int4 v = *reinterpret_cast<const int4 *>(p_rx + tl + 8 * q);
            rh[4 * q + 0] = v.x + (K >> 1);
            rh[4 * q + 1] = v.y + (K >> 1);
            rh[4 * q + 2] = v.z + (K >> 1);
            rh[4 * q + 3] = v.w + (K >> 1);
        }
        if (fast) {
            char *y_blk = reinterpret_cast<char *>(Y + (size_t)(t0 + tl) * N + n0 + nl);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int a4 = qb_a4(acc[r], rx[r]);
                __builtin_nontemporal_store(asym_value(a4, rh[r], asym_L, hr[r], dn, zn) + bv,
                                            reinterpret_cast<float *>(y_blk + (size_t)(8 * (r >> 2) + (r & 3)) * N * 4));
            }
        } else if (n0 + nl < N) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int t = t0 + tl + 8 * (r >> 2) + (r & 3);
                if (t < T) {
                    const int a4 = qb_a4(acc[r], rx[r]);
                    const size_t at = (size_t)t * N + n0 + nl;
                    Y[at] = asym_value(a4, rh[r], asym_L, hr[r], dn, zn) + bv;
                    if (A4out) A4out[at] = a4;
                }
            }
        }
        return;
    }
    if (fast) {
        char *y_blk = reinterpret_cast<char *>(Y + (size_t)(t0 + tl) * N + n0 + nl);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int a4 = qb_a4(acc[r], rx[r]);
            __builtin_nontemporal_store(sc[r] * (float)a4 + bv,
                                        reinterpret_cast<float *>(y_blk + (size_t)(8 * (r >> 2) + (r & 3)) * N * 4));
        }
    } else if (n0 + nl < N) {  // edge tiles and the debug output: every element checked
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int t = t0 + tl + 8 * (r >> 2) + (r & 3);
            if (t < T) {
                const int a4 = qb_a4(acc[r], rx[r]);
                const size_t at = (size_t)t * N + n0 + nl;
                Y[at] = sc[r] * (float)a4 + bv;
                if (A4out) A4out[at] = a4;
            }
        }
    }
}

// 8-bit output (the next layer's input): where to put it and how to quantize it
struct OutQ {
    int8_t *Yq;       // [T,N] u - 128
    int32_t *rs_y;    // [T] row sums of Yq, accumulated with atomics (zero-filled before the launch)
    float clip_out;   // range [-clip_out, +clip_out]
    int act;          // 0 none, 1 GELU
    const float *hx_rows;  // fp32 output only: one activation scale per token (dynamic range) instead of hx, or null
    const float *q0;       // fp32 output only: asymmetric group ranges (h holds Delta, q0 the lower ends), or null
};

// One linear layer of a launch of the role-split kernel, and the list of them that one launch walks through.
// The workgroups take the tiles of all problems in one sequence (each problem's share padded to a multiple of 8, so
// that the renumbering by XCD stays inside a problem), the copy wavefronts running ahead across problem boundaries
// as they do across tiles: a launch's fixed cost (start, first copies from HBM, drain) is paid once for the list.
struct Problem {
    const int8_t *Xq;
    const int32_t *rs_x;
    const uint8_t *packed;
    const float *h;
    const int32_t *rs_w;
    const float *bias;
    float *Y;
    int32_t *A4out;
    int T, N, K, rows_per_group;
    float hx;
    int tiles_m, tiles_n;
    OutQ oq;
};
constexpr int kMaxGroup = QB_MAX_BATCH;
struct Group {
    int n;                            // problems in the list
    int tile_start[kMaxGroup + 1];    // first tile of problem i in the launch's sequence; [n] = length of the sequence
    Problem p[kMaxGroup];
};
// which problem tile `work` of the sequence belongs to (uniform over the workgroup)
__device__ __forceinline__ int problem_of(const Group &g, int work)
{
    int pi = 0;
    while (pi + 1 < g.n && work >= g.tile_start[pi + 1]) ++pi;
    return pi;
}
// Tile `local` of a problem with nwg = tiles_m*tiles_n tiles -> its number in row-major order, or -1 for a padding
// slot.  Workgroups are dealt to the 8 XCDs in turn; XCD x gets a contiguous range of tiles (n fastest), so that a
// token panel is fetched into one L2 only.
__device__ __forceinline__ int logical_tile(int local, int nwg)
{
    const int xcd = local & 7, idx = local >> 3;
    const int q = nwg >> 3, r = nwg & 7;
    if (idx >= q + (xcd < r ? 1 : 0)) return -1;
    return xcd * q + (xcd < r ? xcd : r) + idx;
}

// One 32x32 block of the 8-bit output: the value that decides the code is formed in binary32 with one
// rounding per step, scale = h_x*h_g, y = scale*float(A4), y = y + bias; then the optional GELU, the clamp to
// the output range and the activation quantizer.  The bytes go to the workgroup's staging tile in LDS
// (BM rows of BN bytes), from where whole rows are written out.  Lane/register roles as in store_block_lds.
template <int BM, int BN, int BNT>
__device__ __forceinline__ void quant_block_lds(const v16i &acc, const uint8_t *pp, int e2, int tl, int nl, int K,
                                                float hx, bool has_bias, const Quantizer &qo, int act,
                                                uint8_t *stg)
{
    // (this file is compiled with -ffp-contract=off: y = scale*float(A4) and y + bias are two roundings)
    asm volatile("" : "+v"(tl));
    const int *p_rx = reinterpret_cast<const int *>(pp);
    const int *p_rw = p_rx + BM;
    const float *p_h = reinterpret_cast<const float *>(p_rw + BN), *p_b = p_h + BN;
    const int coln = 2 * p_rw[nl] + K;
    const float scale = hx * p_h[nl];
    const float bv = has_bias ? p_b[nl] : 0.0f;  // y + 0 = y: the code is the same as without a bias
    const float c = qo.m;
    float y[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int4 v = *reinterpret_cast<const int4 *>(p_rx + tl + 8 * q);
        const int rx[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) y[4 * q + i] = scale * (float)qb_a4(acc[4 * q + i], qb_mad24(e2, rx[i], coln)) + bv;  // |rs_x| < 2^23
    }
    if (act == 1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) y[r] = 0.5f * y[r] * (1.0f + erff(y[r] * 0.70710678118654752f));
    }
    // The quantizer (same steps as Quantizer::code_f) without a branch per element: the reciprocal route for
    // all sixteen, and the true division for all sixteen if any lane's product came too close to a rounding
    // boundary (about one block in five) or the range is too extreme for the reciprocal.
    float s[16], rr[16];
    bool redo = !qo.fast;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        s[r] = __builtin_amdgcn_fmed3f(y[r], -c, c) + c;
        const float tp = s[r] * qo.rinv;
        rr[r] = rintf(tp);
        redo |= !(fabsf(tp - rr[r]) <= 0.4999f);
    }
    if (__any(redo)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) rr[r] = rintf(__fdiv_rn(s[r], qo.delta));
    }
#pragma unroll
    for (int r = 0; r < 16; ++r)
        stg[(tl + 8 * (r >> 2) + (r & 3)) * BNT + nl] = (uint8_t)(uint32_t)rr[r];  // the code u; u - 128 is formed on the way out
}

// ---------------------------------------------------------------------------------------------
// Main kernel (K a multiple of 128): the same data path as above with the work split by role.
//   consumer wavefronts (WM x WN of them): LDS fragment reads, code expansion, MFMA, epilogue
//   producer wavefronts (NPROD): nothing but the global -> LDS copies and the waiting for them
// A copy instruction keeps the issuing wavefront busy for tens of cycles while the texture path
// accepts its 64 addresses; issued from an MFMA wavefront that time is lost to the matrix cores,
// issued from a producer it is free.  Producers also run ahead across tiles: while the consumers
// write tile i out, the first stages of tile i+1 are already being filled.
// Protocol per tile (n steps, ring of NSTAGE stages, copies run D = NSTAGE-1 steps ahead); every
// wavefront executes exactly n+1 barriers:
//   producer: start copies 0..D-1; wait copy 0; BARRIER;
//             for s: start copy s+D (its stage was read in step s-1, finished at the last barrier);
//                    wait copy s+1 (vmcnt leaves the younger ones in flight); BARRIER
//   consumer: BARRIER; for s: MMA on stage s % NSTAGE; wait until the stage's LDS reads have returned; BARRIER
// OUTQ: instead of Y the tile is quantized to 8 bits (quant_block_lds) into an LDS staging tile and, after one
// more barrier per tile (E, executed by the producers once the next tile's first copies are on their way), written
// out in whole rows; the rows' sums are collected in LDS and added to rs_y one tile later.
// OUT: 0 fp32 Y, 1 the 8-bit output (OUTQ), 2 fp32 Y from asymmetric group ranges (ASYM; a variant of its own so
// that the others carry none of its code)
template <int BITS, int TM, int TN, int WM, int WN, int NSTAGE, int NPROD, bool SIMD3, int OUT>
__global__ __launch_bounds__(64 * (WM * WN + NPROD), (SIMD3 && OUT != 2 && NSTAGE == 2) ? 4 : 2) void qgemm_i8_ws_kernel(const Group g)
{
    constexpr bool OUTQ = OUT == 1, ASYM = OUT == 2;
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "ring of 2..4 stages");
    constexpr int NC = WM * WN;
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 128;
    constexpr int SLOT = 4 * BITS;                  // bytes per slot in memory
    constexpr int CH = (BITS == 3) ? 12 : 16;       // bytes one lane moves per weight copy instruction
    constexpr int LSLOT = (BITS == 3) ? 16 : SLOT;  // a 12-byte copy lands at a 16-byte stride in LDS
    constexpr int PAIR = 128 * SLOT;                // one 32-neuron block x two units, contiguous in memory
    constexpr int LPAIR = 128 * LSLOT;
    constexpr int PARTS = PAIR / (64 * CH);         // copy instructions per pair; each fills 1024 bytes of LDS
    constexpr int A_TOTAL = BM / 8, B_TOTAL = (BN / 32) * PARTS;  // copy instructions per step
    constexpr int A_PER = (A_TOTAL + NPROD - 1) / NPROD, B_PER = (B_TOTAL + NPROD - 1) / NPROD;
    constexpr int PERP = A_PER + B_PER;             // per producer and step
    constexpr int D = NSTAGE - 1;
    constexpr int A_BYTES = BM * BK, B_BYTES = (BN / 32) * LPAIR, STAGE_BYTES = A_BYTES + B_BYTES;
    static_assert((D - 1) * PERP + 2 * (BM / 64) + 4 * ((BN + 63) / 64) < 64, "vmcnt has six bits");
    constexpr int BNP = (BN + 63) / 64 * 64;        // per-neuron parameter arrays are filled 64 entries at a time
    // rs_x | rs_w | h of the neuron's group | bias | per-token scales | q0 of the neuron's group (asymmetric ranges)
    constexpr int PARAM_BYTES = (2 * BM + (OUT == 2 ? 4 : 3) * BNP) * 4;
    static_assert(!SIMD3 || (NC == 6 && NPROD == 2), "SIMD3: six MFMA wavefronts on SIMDs 0..2, two copy wavefronts on SIMD 3");

    // A tile's parameter block is read in its write-out, which ends before the consumers pass the first
    // barrier of the next tile; the producer rewrites the block two tiles later, after the next tile's
    // last barrier.  Hence two blocks.
    constexpr int NPARAM = 2;

    constexpr int STG_OFF = NSTAGE * STAGE_BYTES + NPARAM * PARAM_BYTES;  // staging tile, then BM row sums
    constexpr int STG_BYTES = OUTQ ? BM * BN + BM * 4 : 0;
    static_assert(STG_OFF % 16 == 0 && BN % 16 == 0 && BM <= NC * 64, "staging tile: 16-byte pieces, one thread per row sum");
    __shared__ __align__(1024) uint8_t lds[STG_OFF + STG_BYTES];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nseq = g.tile_start[g.n];  // tiles (and padding slots) of all problems of the launch

    // Roles.  The wavefronts of a workgroup are dealt to the four SIMDs of the CU in turn (wavefront w runs
    // on SIMD w%4), and a global load or global -> LDS copy issued on a SIMD that is busy with 32x32 MFMAs
    // runs at about half speed (and slows the MFMAs), while one issued on a SIMD without MFMAs does not.
    // SIMD3 layout: wavefronts 3 and 7 copy, the other six multiply, so that three SIMDs run MFMAs at
    // full rate and the fourth feeds them.  (Roles depend on the wavefront number only: a different
    // placement by the hardware would cost speed, not correctness.)
    const bool is_producer = SIMD3 ? (wave & 3) == 3 : wave >= NC;
    if (is_producer) {
        // ================================ producer ================================
        const int p = SIMD3 ? wave >> 2 : wave - NC;
        int pb = 0;
        bool had_tile = false;
        for (int work = blockIdx.x; work < nseq; work += gridDim.x) {
            const int pi = problem_of(g, work);
            const Problem &P = g.p[pi];
            const int logical = logical_tile(work - g.tile_start[pi], P.tiles_m * P.tiles_n);
            if (logical < 0) continue;  // padding slot (the consumers skip it as well)
            const int T = P.T, N = P.N, K = P.K, rows_per_group = P.rows_per_group;
            const int8_t *__restrict__ Xq = P.Xq;
            const int32_t *__restrict__ rs_x = P.rs_x, *__restrict__ rs_w = P.rs_w;
            const uint8_t *__restrict__ packed = P.packed;
            const float *__restrict__ h = P.h, *__restrict__ bias = P.bias;
            const OutQ &oq = P.oq;
            const int nsteps = K / BK, kunits = K >> 6, ncb = (N + 31) >> 5;
            const int tile_m = logical / P.tiles_n, tile_n = logical - tile_m * P.tiles_n;
            // token rows: lane l of a copy fills physical chunk l%8 of row l/8 of an 8-row block; the
            // chunk holds logical chunk (l%8) ^ ((row/2)%8): the swizzle that makes 16 consecutive
            // rows of one logical chunk land in 16 different 16-byte bank groups
            const int last_row = T - 1 - tile_m * BM;  // rows past the end re-read the last one; outputs masked
            // addresses: a wavefront-uniform base per tile and step, a 32-bit byte offset per lane and copy
            const int8_t *a_base = Xq + (size_t)tile_m * BM * K;
            uint32_t a_off[A_PER], a_dst[A_PER];
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                const int blk = (i * NPROD + p) % A_TOTAL;  // surplus copies repeat one: same bytes, same place
                int row = blk * 8 + (lane >> 3);
                const int key = (row >> 1) & 7;
                row = row < last_row ? row : last_row;
                a_off[i] = (uint32_t)row * (uint32_t)K + (((lane & 7) ^ key) * 16);
                a_dst[i] = blk * 1024;
            }
            const int cb0 = tile_n * (BN / 32);
            const uint8_t *b_base = packed + (size_t)cb0 * kunits * 64 * SLOT;
            uint32_t b_off[B_PER], b_dst[B_PER];
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int j = (i * NPROD + p) % B_TOTAL;
                const int pair = j / PARTS, part = j - pair * PARTS;
                int cb = cb0 + pair;
                cb = cb < ncb ? cb : ncb - 1;  // blocks past the end re-read the last one; outputs masked
                b_off[i] = (uint32_t)(cb - cb0) * (uint32_t)(kunits * 64 * SLOT) + part * 64 * CH + lane * CH;
                b_dst[i] = A_BYTES + pair * LPAIR + part * 1024;
            }
            auto fetch = [&](int step, int stage) {
                const uint32_t st_ = lds_base + stage * STAGE_BYTES;
                const uint8_t *bs = b_base + (size_t)step * PAIR;
                const int8_t *as = a_base + (size_t)step * BK;
#pragma unroll
                for (int i = 0; i < B_PER; ++i) {
                    if constexpr (BITS == 3) copy12_to_lds(bs, b_off[i], st_ + b_dst[i]);
                    else copy16_to_lds(bs, b_off[i], st_ + b_dst[i]);
                }
#pragma unroll
                for (int i = 0; i < A_PER; ++i) copy16_to_lds(as, a_off[i], st_ + a_dst[i]);
            };
            if (0 < nsteps) fetch(0, 0);  // the first step's copies go first: the K-loop waits for nothing else
            if (p == 0) {  // the tile's epilogue parameters: needed after the K-loop only
                const uint32_t pbase = lds_base + NSTAGE * STAGE_BYTES + pb * PARAM_BYTES;
#pragma unroll
                for (int c = 0; c < BM / 64; ++c) {
                    int t = tile_m * BM + c * 64 + lane;
                    t = t < T ? t : T - 1;
                    copy4_to_lds(rs_x + t, pbase + c * 256);
                    if (oq.hx_rows) copy4_to_lds(oq.hx_rows + t, pbase + (BM + 3 * BNP) * 4 + c * 256);
                }
#pragma unroll
                for (int c = 0; c < BNP / 64; ++c) {
                    int n = tile_n * BN + c * 64 + lane;
                    n = n < N ? n : N - 1;
                    copy4_to_lds(rs_w + n, pbase + BM * 4 + c * 256);
                    copy4_to_lds(h + n / rows_per_group, pbase + (BM + BNP) * 4 + c * 256);
                    if (bias) copy4_to_lds(bias + n, pbase + (BM + 2 * BNP) * 4 + c * 256);
                    if constexpr (ASYM) copy4_to_lds(oq.q0 + n / rows_per_group, pbase + (2 * BM + 3 * BNP) * 4 + c * 256);
                }
            }
            pb ^= 1;
#pragma unroll
            for (int u = 1; u < D; ++u)
                if (u < nsteps) fetch(u, u);
            if (OUTQ && had_tile) __builtin_amdgcn_s_barrier();  // barrier E of the previous tile
            had_tile = true;
            // step 0 has landed when only younger copies are outstanding: steps 1..D-1 and, in the wavefront
            // that issued them, the parameter copies (their number depends on bias and per-token scales)
            if (nsteps >= D) {
                constexpr int W0 = (D - 1) * PERP, PM = BM / 64, PN = BNP / 64;
                constexpr int PA = ASYM ? PN : 0;
                if (p != 0) wait_vmcnt<W0>();
                else if (oq.hx_rows) { if (bias) wait_vmcnt<W0 + 2 * PM + 3 * PN + PA>(); else wait_vmcnt<W0 + 2 * PM + 2 * PN + PA>(); }
                else { if (bias) wait_vmcnt<W0 + PM + 3 * PN + PA>(); else wait_vmcnt<W0 + PM + 2 * PN + PA>(); }
            } else {
                wait_vmcnt<0>();
            }
            __builtin_amdgcn_s_barrier();
            int stage = D % NSTAGE;  // stage of step s + D
            for (int s = 0; s < nsteps; ++s) {
                if (s + D < nsteps) {
                    fetch(s + D, stage);
                    wait_vmcnt<(D - 1) * PERP>();
                } else {
                    wait_vmcnt<0>();
                }
                stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
                __builtin_amdgcn_s_barrier();
            }
        }
        if (OUTQ && had_tile) __builtin_amdgcn_s_barrier();  // barrier E of the last tile
        return;
    }

    // ================================ consumer ================================
    const int cidx = SIMD3 ? (wave & 3) + 3 * (wave >> 2) : wave;
    const int wm = cidx / WN, wn = cidx - wm * WN;
    const int l32 = lane & 31, hf = lane >> 5;
    // token fragments: row = wm*TM*32 + tm*32 + l32, logical chunk = kk*4 + hf*2 + sub
    const int p0 = (hf * 2) ^ ((l32 >> 1) & 7);
    const int frag_row = (wm * TM * 32 + l32) * BK;
    int a_frag[4];
    a_frag[0] = frag_row + ((p0 ^ 0) << 4);  // kk 0, sub 0
    a_frag[1] = frag_row + ((p0 ^ 1) << 4);  // kk 0, sub 1
    a_frag[2] = frag_row + ((p0 ^ 4) << 4);  // kk 1, sub 0
    a_frag[3] = frag_row + ((p0 ^ 5) << 4);  // kk 1, sub 1
    const int b_frag = A_BYTES + wn * TN * LPAIR + lane * LSLOT;  // + tn*LPAIR + kk*64*LSLOT
    constexpr int L = (1 << BITS) - 1;
    constexpr int E2 = (BITS == 8) ? 2 : -2 * L;  // 2*e
    int pb = 0;

    v16i acc[TM][TN];

    // 8-bit output: staging tile, row sums, the output quantizer
    constexpr int NCT = NC * 64;
    const int ctid = cidx * 64 + lane;
    uint8_t *stg = lds + STG_OFF;
    int *rowsum = reinterpret_cast<int *>(lds + STG_OFF + BM * BN);
    Quantizer qo;
    int prev_t0 = -1, prev_T = 0;  // the tile whose row sums still sit in LDS, and its problem's token count and rs_y
    int32_t *prev_rs_y = nullptr;
    if constexpr (OUTQ) {
        if (ctid < BM) rowsum[ctid] = 0;
    }
    auto flush_rowsums = [&]() {  // the previous tile's row sums -> rs_y; every LDS add to them is a barrier back
        if (ctid < BM) {
            const int v = rowsum[ctid];
            rowsum[ctid] = 0;
            if (prev_t0 + ctid < prev_T) atomicAdd(prev_rs_y + prev_t0 + ctid, v);
        }
    };

    for (int work = blockIdx.x; work < nseq; work += gridDim.x) {
        const int pi = problem_of(g, work);
        const Problem &P = g.p[pi];
        const int logical = logical_tile(work - g.tile_start[pi], P.tiles_m * P.tiles_n);
        if (logical < 0) continue;  // padding slot (the producers skip it as well)
        const int T = P.T, N = P.N, K = P.K;
        const float hx = P.hx;
        const float *__restrict__ bias = P.bias;
        float *__restrict__ Y = P.Y;
        int32_t *__restrict__ A4out = P.A4out;
        const OutQ &oq = P.oq;
        const int nsteps = K / BK;
        const int tile_m = logical / P.tiles_n, tile_n = logical - tile_m * P.tiles_n;
        if constexpr (OUTQ) qo.set(oq.clip_out, 255.0f);

#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0;

// One step: every LDS read of the step is issued first (12 reads in flight, their latency paid once),
// then the 16 MFMAs run while the later reads are still arriving.  The scheduling barrier keeps the
// compiler from folding the reads back into a read-wait-multiply chain.
#define QB_MMA(stage)                                                                                     \
    {                                                                                                     \
        const uint8_t *st_ = lds + (stage) * STAGE_BYTES;                                                 \
        uint32_t raw[2][TN][BITS];                                                                        \
        v4i afr[2][2][TM];                                                                                \
        _Pragma("unroll") for (int kk = 0; kk < 2; ++kk) {                                                \
            _Pragma("unroll") for (int tn = 0; tn < TN; ++tn)                                             \
                SlotRead<BITS>::get(st_ + b_frag + tn * LPAIR + kk * 64 * LSLOT, raw[kk][tn]);            \
            _Pragma("unroll") for (int sub = 0; sub < 2; ++sub)                                           \
                _Pragma("unroll") for (int tm = 0; tm < TM; ++tm) afr[kk][sub][tm] =                      \
                    *reinterpret_cast<const v4i *>(st_ + a_frag[kk * 2 + sub] + tm * 32 * BK);            \
        }                                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        _Pragma("unroll") for (int kk = 0; kk < 2; ++kk) {                                                \
            uint32_t d[TN][8];                                                                            \
            _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) {                                           \
                unpack_run<BITS>(raw[kk][tn], d[tn]);                                                     \
                if constexpr (BITS == 8) {                                                                \
                    _Pragma("unroll") for (int i = 0; i < 8; ++i) d[tn][i] ^= 0x80808080u;                \
                }                                                                                         \
            }                                                                                             \
            _Pragma("unroll") for (int sub = 0; sub < 2; ++sub) {                                         \
                v4i b[TN];                                                                                \
                _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) {                                       \
                    b[tn][0] = (int)d[tn][4 * sub + 0];                                                   \
                    b[tn][1] = (int)d[tn][4 * sub + 1];                                                   \
                    b[tn][2] = (int)d[tn][4 * sub + 2];                                                   \
                    b[tn][3] = (int)d[tn][4 * sub + 3];                                                   \
                }                                                                                         \
                _Pragma("unroll") for (int tm = 0; tm < TM; ++tm)                                         \
                    _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) acc[tm][tn] =                       \
                        __builtin_amdgcn_mfma_i32_32x32x32_i8(afr[kk][sub][tm], b[tn], acc[tm][tn], 0, 0, 0); \
            }                                                                                             \
        }                                                                                                 \
    }
// a bare barrier (no fence: the producers' vmcnt wait is what makes the copies visible); the empty
// asm keeps the compiler from moving LDS reads across it.  The wait for the LDS counter in front of it: the
// stage just read is overwritten by copies that the producers start right behind the barrier, so this
// wavefront's reads of it must have returned, not only been issued (the compiler lets the MFMAs that consume
// the step's last fragments follow below the barrier).
#define QB_BARRIER()                                                                                      \
    {                                                                                                     \
        __builtin_amdgcn_s_waitcnt(0xC07F); /* lgkmcnt(0) */                                              \
        asm volatile("" ::: "memory");                                                                    \
        __builtin_amdgcn_s_barrier();                                                                     \
        asm volatile("" ::: "memory");                                                                    \
    }

        if constexpr (OUTQ) __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): my LDS writes and adds are done
        QB_BARRIER()
        if constexpr (OUTQ) {
            if (prev_t0 >= 0) flush_rowsums();
        }
        int s = 0;
        for (; s + NSTAGE <= nsteps; s += NSTAGE) {
#pragma unroll
            for (int u = 0; u < NSTAGE; ++u) {
                QB_MMA(u)
                QB_BARRIER()
            }
        }
#pragma unroll
        for (int u = 0; u < NSTAGE - 1; ++u)
            if (s + u < nsteps) {
                QB_MMA(u)
                QB_BARRIER()
            }
#undef QB_MMA

        // ---- write-out
        if constexpr (OUTQ) {
            typedef unsigned int v4u __attribute__((ext_vector_type(4)));
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    quant_block_lds<BM, BNP, BN>(acc[tm][tn], lds + NSTAGE * STAGE_BYTES + pb * PARAM_BYTES, E2,
                                                 (wm * TM + tm) * 32 + 4 * hf, (wn * TN + tn) * 32 + l32, K, hx,
                                                 bias != nullptr, qo, oq.act, stg);
            __builtin_amdgcn_s_waitcnt(0xC07F);  // the staging bytes are written
            QB_BARRIER()                         // barrier E
            // whole rows out: 16-byte pieces, BN/16 per row
            constexpr int PPR = BN / 16;
            const int t0 = tile_m * BM, n0 = tile_n * BN;
            const bool vec_ok = (N & 15) == 0 && (reinterpret_cast<uintptr_t>(oq.Yq) & 15) == 0;
            for (int pc = ctid; pc < BM * PPR; pc += NCT) {
                const int row = pc / PPR, cp = pc - row * PPR;
                const int t = t0 + row, n = n0 + cp * 16;
                if (t < T && n < N) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * BN + cp * 16);  // codes u
                    int8_t *dst = oq.Yq + (size_t)t * N + n;
                    int sum;
                    if (vec_ok && n + 16 <= N) {
                        v4u o = {v.x ^ 0x80808080u, v.y ^ 0x80808080u, v.z ^ 0x80808080u, v.w ^ 0x80808080u};  // u - 128
                        __builtin_nontemporal_store(o, reinterpret_cast<v4u *>(dst));
                        uint32_t su = __builtin_amdgcn_sad_u8(v.x, 0u, 0u);
                        su = __builtin_amdgcn_sad_u8(v.y, 0u, su);
                        su = __builtin_amdgcn_sad_u8(v.z, 0u, su);
                        su = __builtin_amdgcn_sad_u8(v.w, 0u, su);
                        sum = (int)su - 16 * 128;
                    } else {
                        const uint32_t w[4] = {v.x ^ 0x80808080u, v.y ^ 0x80808080u, v.z ^ 0x80808080u, v.w ^ 0x80808080u};
                        sum = 0;
#pragma unroll
                        for (int b = 0; b < 16; ++b)
                            if (n + b < N) {
                                const int8_t q8 = (int8_t)((w[b >> 2] >> (8 * (b & 3))) & 255u);
                                dst[b] = q8;
                                sum += q8;
                            }
                    }
                    atomicAdd(rowsum + row, sum);
                }
            }
            prev_t0 = t0;
            prev_T = T;
            prev_rs_y = oq.rs_y;
        } else {
        const bool fast = (tile_m + 1) * BM <= T && (tile_n + 1) * BN <= N && A4out == nullptr;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                store_block_lds<BM, BNP>(acc[tm][tn], lds + NSTAGE * STAGE_BYTES + pb * PARAM_BYTES, E2,
                                        (wm * TM + tm) * 32 + 4 * hf, (wn * TN + tn) * 32 + l32, tile_m * BM, tile_n * BN,
                                        T, N, K, hx, bias != nullptr, fast, Y, A4out, oq.hx_rows != nullptr,
                                        ASYM ? L : 0);
        }
        pb ^= 1;
    }
    if constexpr (OUTQ) {
        if (prev_t0 >= 0) {  // the last tile's row sums: the producers have left, the six MFMA wavefronts meet once more
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
            flush_rowsums();
        }
    }
#undef QB_BARRIER
}

// Adds one problem to a launch list of the role-split kernel with BM x BN tiles; false when the list is full.
template <int BM, int BN>
bool group_add(Group &g, const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
               const float *bias, float *Y, int32_t *A4, int T, int N, int K, int rpg, float hx, const OutQ &oq)
{
    if (g.n >= kMaxGroup) return false;
    Problem &P = g.p[g.n];
    P.Xq = Xq; P.rs_x = rs_x; P.packed = packed; P.h = h; P.rs_w = rs_w; P.bias = bias; P.Y = Y; P.A4out = A4;
    P.T = T; P.N = N; P.K = K; P.rows_per_group = rpg; P.hx = hx;
    P.tiles_m = (T + BM - 1) / BM;
    P.tiles_n = (N + BN - 1) / BN;
    P.oq = oq;
    const int nwg = P.tiles_m * P.tiles_n;
    if (g.n == 0) g.tile_start[0] = 0;
    // a problem's share of the sequence is padded to a multiple of 8 (the last one needs no padding)
    g.tile_start[g.n] = (g.tile_start[g.n] + 7) & ~7;
    g.tile_start[g.n + 1] = g.tile_start[g.n] + nwg;
    ++g.n;
    return true;
}

// One launch for the whole list: a persistent grid of at most grid_cap workgroups (a multiple of 8).
template <int BITS, int TM, int TN, int WM, int WN, int NSTAGE, int NPROD, bool SIMD3, int OUT>
void launch_group(const Group &g, hipStream_t st, int grid_cap)
{
    int grid = g.tile_start[g.n];
    if (grid_cap > 0 && grid > grid_cap) grid = grid_cap;
    hipLaunchKernelGGL((qgemm_i8_ws_kernel<BITS, TM, TN, WM, WN, NSTAGE, NPROD, SIMD3, OUT>), dim3(grid),
                       dim3(64 * (WM * WN + NPROD)), 0, st, g);
}

template <int BITS, int TM, int TN, int WM, int WN, int NSTAGE, int NPROD, bool SIMD3 = false>
void launch_ws(const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
               const float *bias, float *Y, int32_t *A4, int T, int N, int K, int rpg, float hx, hipStream_t st,
               int grid_cap, const float *hx_rows = nullptr, const float *q0 = nullptr)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    const OutQ oq{nullptr, nullptr, 1.0f, 0, hx_rows, q0};
    Group g;
    g.n = 0;
    group_add<BM, BN>(g, Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, oq);
    if (q0) launch_group<BITS, TM, TN, WM, WN, NSTAGE, NPROD, SIMD3, 2>(g, st, grid_cap);
    else launch_group<BITS, TM, TN, WM, WN, NSTAGE, NPROD, SIMD3, 0>(g, st, grid_cap);
}

// the same with the 8-bit output
template <int BITS, int TM, int TN, int WM, int WN, int NSTAGE, int NPROD, bool SIMD3 = false>
void launch_ws_q8(const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
                  const float *bias, const OutQ &oq, int T, int N, int K, int rpg, float hx, hipStream_t st, int grid_cap)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    Group g;
    g.n = 0;
    group_add<BM, BN>(g, Xq, rs_x, packed, h, rs_w, bias, nullptr, nullptr, T, N, K, rpg, hx, oq);
    launch_group<BITS, TM, TN, WM, WN, NSTAGE, NPROD, SIMD3, 1>(g, st, grid_cap);
}

template <int BITS, int TM, int TN, int WM, int WN, int KU>
void launch_cfg(const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
                const float *bias, float *Y, int32_t *A4, int T, int N, int K, int rpg, float hx, hipStream_t st,
                const float *hx_rows = nullptr, const float *q0 = nullptr)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL((qgemm_i8_kernel<BITS, TM, TN, WM, WN, KU>), dim3(tiles_m * tiles_n), dim3(64 * WM * WN), 0, st,
                       Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, tiles_m, tiles_n, hx_rows, q0);
}

// grid_cap: upper bound of workgroups (a multiple of 8); 0 = one workgroup per tile
template <int BITS, int TM, int TN, int WM, int WN, int NSTAGE>
void launch_dma(const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
                const float *bias, float *Y, int32_t *A4, int T, int N, int K, int rpg, float hx, hipStream_t st,
                int grid_cap = 0)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    int grid = tiles_m * tiles_n;
    if (grid_cap > 0 && grid > grid_cap) grid = grid_cap;
    hipLaunchKernelGGL((qgemm_i8_dma_kernel<BITS, TM, TN, WM, WN, NSTAGE>), dim3(grid), dim3(64 * WM * WN), 0, st,
                       Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, tiles_m, tiles_n);
}

template <int BITS>
void launch_bits(const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
                 const float *bias, float *Y, int32_t *A4, int T, int N, int K, int rpg, float hx, hipStream_t st,
                 const float *hx_rows = nullptr, const float *q0 = nullptr)
{
    const long tiles128 = (long)((T + 127) / 128) * ((N + 127) / 128);
    if (tiles128 <= 160) {
        // Few tiles (small token counts, the inference regime): the persistent kernels below leave most CUs idle
        // and pay ~6.5 us at least; 32x64 tiles of the register-staged kernel spread the work over the chip
        // (measured 4.4-5 us against 8 at T <= 1024, N = 768; 6.8 against 8.4 at 1024 x 2304 x 768; equal
        // at about 190 tiles).  Long contractions take 256 features per step.
        if (K % 256 == 0 && K >= 2048) launch_cfg<BITS, 1, 1, 1, 2, 4>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st, hx_rows, q0);
        else if (K % 128 == 0) launch_cfg<BITS, 1, 1, 1, 2, 2>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st, hx_rows, q0);
        else launch_cfg<BITS, 1, 1, 1, 2, 1>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st, hx_rows, q0);
        return;
    }
    if (K % 128 != 0) {  // odd number of 64-feature units: register-staged kernel, one unit per step
        launch_cfg<BITS, 2, 2, 2, 2, 1>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st, hx_rows, q0);
        return;
    }
    // Tile choice (measured on BERT-base and BERT-large shapes).  Copies issued on a SIMD that is busy
    // with 32x32 MFMAs run at about half their stand-alone rate, so where the tile count allows it the MFMAs
    // go to three SIMDs and the copies to the fourth:
    //   128x96 tiles in that layout when they need fewer rounds over the 256 CUs than 128x128 tiles would,
    //     weighted by the measured cost of a tile (0.86 of a 128x128 one): all of BERT-base's N = 768 layers
    //     at 4096 and 12288 tokens, and N = 2304 at 4096;
    //   else 128x128: the role-split kernel (one workgroup per CU, copies run ahead across tiles) when a CU
    //     gets few tiles or the contraction is long and the tiles are few, two plain workgroups per CU when
    //     it gets many (one's write-out overlaps the other's MFMAs); this also beats 256x256 tiles on the
    //     BERT-large shapes at 32768 tokens (2.3 against 2.07 POP/s at 2 bits).
    // Grids are persistent and a multiple of 8, so that a workgroup stays inside its XCD's tile range.
    const long tiles96 = (long)((T + 127) / 128) * ((N + 95) / 96);
    const long rounds128 = (tiles128 + 255) / 256, rounds96 = (tiles96 + 255) / 256;
    // (also where 128x128 tiles would need fewer rounds, for up to five rounds of 128x96 tiles: as two workgroups per CU
    // they are 3 % ahead of the plain two-workgroup kernel on BERT-base's FFN-up)
    if (86 * rounds96 < 100 * rounds128 || (N % 96 == 0 && tiles96 > 256 && tiles96 <= 1280))
    {
        // more tiles than CUs: two workgroups per CU, one's write-out under the other's K-loop (LDS and registers allow it
        // at 2, 3 and 4 bits; at 8 bits with two stages, for the plain fp32 output)
        if (tiles96 > 256 && BITS < 8) launch_ws<BITS, 2, 1, 2, 3, 3, 2, true>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st, 512, hx_rows, q0);
        else if (tiles96 > 256 && !q0) launch_ws<BITS, 2, 1, 2, 3, 2, 2, true>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st, 512, hx_rows, q0);
        else launch_ws<BITS, 2, 1, 2, 3, 3, 2, true>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st, 256, hx_rows, q0);
    }
    else if (hx_rows || q0 || tiles128 <= 640 || (K >= 2048 && tiles128 <= 1024))  // (per-token scales, asymmetric ranges: role-split kernels only)
        launch_ws<BITS, 2, 2, 2, 2, 3, 4>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st, 256, hx_rows, q0);
    else
        launch_dma<BITS, 2, 2, 2, 2, 2>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st, 512);
}

// 8-bit output: the role-split kernels only (128x96 tiles on three SIMDs where they need fewer rounds, else 128x128)
template <int BITS>
void launch_bits_q8(const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
                    const float *bias, const OutQ &oq, int T, int N, int K, int rpg, float hx, hipStream_t st)
{
    const long tiles128 = (long)((T + 127) / 128) * ((N + 127) / 128);
    const long tiles96 = (long)((T + 127) / 128) * ((N + 95) / 96);
    const long rounds128 = (tiles128 + 255) / 256, rounds96 = (tiles96 + 255) / 256;
    if (86 * rounds96 < 100 * rounds128 || (N % 96 == 0 && tiles96 > 256)) {
        // more tiles than CUs: two stages, so that two workgroups fit a CU and one's output quantizer runs under the
        // other's K-loop (then also where 128x128 tiles would need fewer rounds)
        if (tiles96 > 256) launch_ws_q8<BITS, 2, 1, 2, 3, 2, 2, true>(Xq, rs_x, packed, h, rs_w, bias, oq, T, N, K, rpg, hx, st, 512);
        else launch_ws_q8<BITS, 2, 1, 2, 3, 3, 2, true>(Xq, rs_x, packed, h, rs_w, bias, oq, T, N, K, rpg, hx, st, 256);
    } else
        launch_ws_q8<BITS, 2, 2, 2, 2, 3, 4>(Xq, rs_x, packed, h, rs_w, bias, oq, T, N, K, rpg, hx, st, 256);
}

__global__ void fill_zero_i32_kernel(int32_t *p, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

}  // namespace
}  // namespace qb

using namespace qb;

extern "C" qb_status qb_qlinear_fwd(const int8_t *Xq, const int32_t *rs_x, float clip, const void *packed,
                                    const float *h, const int32_t *rs_w, int bits, int groups, int64_t T, int64_t N,
                                    int64_t K, const float *bias, float *Y, int32_t *A4_debug, void *stream)
{
    if (!Xq || !rs_x || !packed || !h || !rs_w || !Y) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (T <= 0 || T > (1 << 24) || N <= 0 || N > (1 << 24) || !k_ok(K) || groups <= 0 || N % groups != 0)
        return QB_ERR_SHAPE;
    if (!(clip > 0.0f) || !(clip < 3.0e38f)) return QB_ERR_CLIP;
    const float hx = clip / 255.0f;
    const int rpg = (int)(N / groups);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t *p = static_cast<const uint8_t *>(packed);
    switch (bits) {
        case 2: launch_bits<2>(Xq, rs_x, p, h, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, hx, st); break;
        case 3: launch_bits<3>(Xq, rs_x, p, h, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, hx, st); break;
        case 4: launch_bits<4>(Xq, rs_x, p, h, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, hx, st); break;
        default: launch_bits<8>(Xq, rs_x, p, h, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, hx, st); break;
    }
    return launch_status();
}

namespace {
qb_status check_fwd_job(const qb_fwd_job &j)
{
    if (!j.Xq || !j.rs_x || !j.packed || !j.h || !j.rs_w || !j.Y) return QB_ERR_NULL;
    if (!bits_ok(j.bits)) return QB_ERR_BITS;
    if (j.T <= 0 || j.T > (1 << 24) || j.N <= 0 || j.N > (1 << 24) || !k_ok(j.K) || j.groups <= 0 || j.N % j.groups != 0)
        return QB_ERR_SHAPE;
    if (!(j.clip > 0.0f) || !(j.clip < 3.0e38f)) return QB_ERR_CLIP;
    return QB_OK;
}

template <int BITS>
void launch_job(const qb_fwd_job &j, hipStream_t st)
{
    launch_bits<BITS>(j.Xq, j.rs_x, static_cast<const uint8_t *>(j.packed), j.h, j.rs_w, j.bias, j.Y, nullptr, (int)j.T, (int)j.N,
                      (int)j.K, (int)(j.N / j.groups), j.clip / 255.0f, st);
}

// A shared launch of 128x96 tiles.  Two workgroups per CU (512 resident): while one writes a tile out and starts the
// next, the other's K-loop keeps the matrix cores busy (the step's GEMM stage 196 -> 171 us).  That needs at most
// 80 KB of LDS and 128 registers: three stages at 2, 3 and 4 bits (64-73 KB, 102 registers), two stages at 8 bits.
template <int BITS>
void launch_g96(const Group &g, hipStream_t st)
{
    if (BITS == 8 && g.tile_start[g.n] > 256) launch_group<BITS, 2, 1, 2, 3, 2, 2, true, 0>(g, st, 512);
    else launch_group<BITS, 2, 1, 2, 3, 3, 2, true, 0>(g, st, 512);  // (no more than one workgroup per CU at 8 bits)
}

// the jobs of one bit-width: those that the single call would give to a role-split kernel share launches of it
// (one list per tile shape), the others go one by one
template <int BITS>
void launch_jobs_of_width(const qb_fwd_job *jobs, int n_jobs, hipStream_t st)
{
    Group g96, g128;
    g96.n = g128.n = 0;
    SmallGroup small[3];  // few-tile problems, by features per step (64, 128, 256)
    small[0].n = small[1].n = small[2].n = 0;
    auto flush_small = [&](int c) {
        SmallGroup &sg = small[c];
        if (sg.n == 0) return;
        const dim3 grid(sg.first_wg[sg.n]);
        if (c == 0) hipLaunchKernelGGL((qgemm_i8_small_group_kernel<BITS, 1>), grid, dim3(128), 0, st, sg);
        else if (c == 1) hipLaunchKernelGGL((qgemm_i8_small_group_kernel<BITS, 2>), grid, dim3(128), 0, st, sg);
        else hipLaunchKernelGGL((qgemm_i8_small_group_kernel<BITS, 4>), grid, dim3(128), 0, st, sg);
        sg.n = 0;
    };
    const OutQ none{nullptr, nullptr, 1.0f, 0, nullptr, nullptr};
    for (int i = 0; i < n_jobs; ++i) {
        const qb_fwd_job &j = jobs[i];
        if (j.bits != BITS) continue;
        // the tile choice of the single call (launch_bits): problems it gives to a role-split kernel share launches,
        // the others (few tiles, K not a multiple of 128, many tiles: two plain workgroups per CU) go one by one
        const long tiles128 = (long)((j.T + 127) / 128) * ((j.N + 127) / 128);
        const long tiles96 = (long)((j.T + 127) / 128) * ((j.N + 95) / 96);
        const long rounds128 = (tiles128 + 255) / 256, rounds96 = (tiles96 + 255) / 256;
        const bool few128 = tiles128 <= 640 || (j.K >= 2048 && tiles128 <= 1024);
        // ... except that a problem which alone would run as two plain workgroups per CU joins the 128x96 list when 96
        // divides its N and it has no more than five rounds of tiles: inside a shared launch it pays no start-up of its
        // own and its tiles fill the rounds the other problems leave ragged (BERT-base FFN-up at 4096 tokens: the
        // step's GEMM stage 212 -> 197 us; with twelve and more rounds, at 12288 tokens or BERT-large's 32768, the two
        // workgroups per CU stay 3-5 % ahead)
        const bool use96 = 86 * rounds96 < 100 * rounds128 || (!few128 && j.N % 96 == 0 && tiles96 <= 1280);
        const bool use128 = !use96 && few128;
        if (tiles128 <= 160) {  // few tiles: the 32x64-tile form, the step width of the single call, one launch per width
            const int c = (j.K % 256 == 0 && j.K >= 2048) ? 2 : (j.K % 128 == 0) ? 1 : 0;
            SmallGroup &sg = small[c];
            if (sg.n == QB_MAX_BATCH) flush_small(c);
            if (sg.n == 0) sg.first_wg[0] = 0;
            SmallProblem &sp = sg.p[sg.n];
            sp.Xq = j.Xq; sp.rs_x = j.rs_x; sp.packed = static_cast<const uint8_t *>(j.packed); sp.h = j.h; sp.rs_w = j.rs_w;
            sp.bias = j.bias; sp.Y = j.Y; sp.T = (int)j.T; sp.N = (int)j.N; sp.K = (int)j.K;
            sp.rows_per_group = (int)(j.N / j.groups); sp.hx = j.clip / 255.0f;
            sp.tiles_m = (int)((j.T + 31) / 32); sp.tiles_n = (int)((j.N + 63) / 64);
            sg.first_wg[sg.n + 1] = sg.first_wg[sg.n] + ((sp.tiles_m * sp.tiles_n + 7) & ~7);
            ++sg.n;
            continue;
        }
        if (j.K % 128 != 0 || !(use96 || use128)) {
            launch_job<BITS>(j, st);
            continue;
        }
        const uint8_t *p = static_cast<const uint8_t *>(j.packed);
        const int rpg = (int)(j.N / j.groups);
        const float hx = j.clip / 255.0f;
        if (use96) {
            if (g96.n == kMaxGroup) {
                launch_g96<BITS>(g96, st);
                g96.n = 0;
            }
            group_add<128, 96>(g96, j.Xq, j.rs_x, p, j.h, j.rs_w, j.bias, j.Y, nullptr, (int)j.T, (int)j.N, (int)j.K, rpg, hx, none);
        } else {
            if (g128.n == kMaxGroup) {
                launch_group<BITS, 2, 2, 2, 2, 3, 4, false, 0>(g128, st, 256);
                g128.n = 0;
            }
            group_add<128, 128>(g128, j.Xq, j.rs_x, p, j.h, j.rs_w, j.bias, j.Y, nullptr, (int)j.T, (int)j.N, (int)j.K, rpg, hx, none);
        }
    }
    if (g96.n) launch_g96<BITS>(g96, st);
    if (g128.n) launch_group<BITS, 2, 2, 2, 2, 3, 4, false, 0>(g128, st, 256);
    for (int c = 0; c < 3; ++c) flush_small(c);
}
}  // namespace

extern "C" qb_status qb_qlinear_fwd_batched(const qb_fwd_job *jobs, int n_jobs, void *stream)
{
    if (n_jobs < 0 || (n_jobs > 0 && !jobs)) return QB_ERR_NULL;
    if (n_jobs == 0) return QB_OK;
    for (int i = 0; i < n_jobs; ++i) {
        const qb_status s = check_fwd_job(jobs[i]);
        if (s != QB_OK) return s;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    launch_jobs_of_width<2>(jobs, n_jobs, st);
    launch_jobs_of_width<3>(jobs, n_jobs, st);
    launch_jobs_of_width<4>(jobs, n_jobs, st);
    launch_jobs_of_width<8>(jobs, n_jobs, st);
    return launch_status();
}

extern "C" qb_status qb_qlinear_fwd_q8(const int8_t *Xq, const int32_t *rs_x, float clip, const void *packed,
                                       const float *h, const int32_t *rs_w, int bits, int groups, int64_t T, int64_t N,
                                       int64_t K, const float *bias, int act, float clip_out, int8_t *Yq, int32_t *rs_y,
                                       void *stream)
{
    if (!Xq || !rs_x || !packed || !h || !rs_w || !Yq || !rs_y) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (T <= 0 || T > (1 << 24) || N <= 0 || N > (1 << 24) || !k_ok(K) || K % 128 != 0 || groups <= 0 || N % groups != 0 ||
        (act != 0 && act != 1))
        return QB_ERR_SHAPE;
    if (!(clip > 0.0f) || !(clip < 3.0e38f) || !(clip_out > 0.0f) || !(clip_out < 3.0e38f)) return QB_ERR_CLIP;
    const float hx = clip / 255.0f;
    const int rpg = (int)(N / groups);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t *p = static_cast<const uint8_t *>(packed);
    const OutQ oq{Yq, rs_y, clip_out, act, nullptr, nullptr};
    hipLaunchKernelGGL(fill_zero_i32_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, st, rs_y, (int)T);
    switch (bits) {
        case 2: launch_bits_q8<2>(Xq, rs_x, p, h, rs_w, bias, oq, (int)T, (int)N, (int)K, rpg, hx, st); break;
        case 3: launch_bits_q8<3>(Xq, rs_x, p, h, rs_w, bias, oq, (int)T, (int)N, (int)K, rpg, hx, st); break;
        case 4: launch_bits_q8<4>(Xq, rs_x, p, h, rs_w, bias, oq, (int)T, (int)N, (int)K, rpg, hx, st); break;
        default: launch_bits_q8<8>(Xq, rs_x, p, h, rs_w, bias, oq, (int)T, (int)N, (int)K, rpg, hx, st); break;
    }
    return launch_status();
}

extern "C" qb_status qb_qlinear_fwd_dyn(const int8_t *Xq, const int32_t *rs_x, const float *hx_rows, const void *packed,
                                        const float *h, const int32_t *rs_w, int bits, int groups, int64_t T, int64_t N,
                                        int64_t K, const float *bias, float *Y, int32_t *A4_debug, void *stream)
{
    if (!Xq || !rs_x || !hx_rows || !packed || !h || !rs_w || !Y) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (T <= 0 || T > (1 << 24) || N <= 0 || N > (1 << 24) || !k_ok(K) || groups <= 0 || N % groups != 0)
        return QB_ERR_SHAPE;
    const int rpg = (int)(N / groups);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t *p = static_cast<const uint8_t *>(packed);
    switch (bits) {
        case 2: launch_bits<2>(Xq, rs_x, p, h, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, 0.0f, st, hx_rows); break;
        case 3: launch_bits<3>(Xq, rs_x, p, h, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, 0.0f, st, hx_rows); break;
        case 4: launch_bits<4>(Xq, rs_x, p, h, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, 0.0f, st, hx_rows); break;
        default: launch_bits<8>(Xq, rs_x, p, h, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, 0.0f, st, hx_rows); break;
    }
    return launch_status();
}

extern "C" qb_status qb_qlinear_fwd_asym(const int8_t *Xq, const int32_t *rs_x, float clip, const void *packed,
                                         const float *delta, const float *q0, const int32_t *rs_w, int bits, int groups,
                                         int64_t T, int64_t N, int64_t K, const float *bias, float *Y, int32_t *A4_debug,
                                         void *stream)
{
    if (!Xq || !rs_x || !packed || !delta || !q0 || !rs_w || !Y) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (T <= 0 || T > (1 << 24) || N <= 0 || N > (1 << 24) || !k_ok(K) || groups <= 0 || N % groups != 0)
        return QB_ERR_SHAPE;
    if (!(clip > 0.0f) || !(clip < 3.0e38f)) return QB_ERR_CLIP;
    const int rpg = (int)(N / groups);
    const float hx = clip / 255.0f;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t *p = static_cast<const uint8_t *>(packed);
    switch (bits) {
        case 2: launch_bits<2>(Xq, rs_x, p, delta, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, hx, st, nullptr, q0); break;
        case 3: launch_bits<3>(Xq, rs_x, p, delta, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, hx, st, nullptr, q0); break;
        case 4: launch_bits<4>(Xq, rs_x, p, delta, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, hx, st, nullptr, q0); break;
        default: launch_bits<8>(Xq, rs_x, p, delta, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, hx, st, nullptr, q0); break;
    }
    return launch_status();
}

extern "C" qb_status qb_qlinear_fwd_asym_dyn(const int8_t *Xq, const int32_t *rs_x, const float *hx_rows, const void *packed,
                                             const float *delta, const float *q0, const int32_t *rs_w, int bits, int groups,
                                             int64_t T, int64_t N, int64_t K, const float *bias, float *Y,
                                             int32_t *A4_debug, void *stream)
{
    if (!Xq || !rs_x || !hx_rows || !packed || !delta || !q0 || !rs_w || !Y) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (T <= 0 || T > (1 << 24) || N <= 0 || N > (1 << 24) || !k_ok(K) || groups <= 0 || N % groups != 0)
        return QB_ERR_SHAPE;
    const int rpg = (int)(N / groups);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t *p = static_cast<const uint8_t *>(packed);
    switch (bits) {
        case 2: launch_bits<2>(Xq, rs_x, p, delta, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, 0.0f, st, hx_rows, q0); break;
        case 3: launch_bits<3>(Xq, rs_x, p, delta, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, 0.0f, st, hx_rows, q0); break;
        case 4: launch_bits<4>(Xq, rs_x, p, delta, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, 0.0f, st, hx_rows, q0); break;
        default: launch_bits<8>(Xq, rs_x, p, delta, rs_w, bias, Y, A4_debug, (int)T, (int)N, (int)K, rpg, 0.0f, st, hx_rows, q0); break;
    }
    return launch_status();
}
