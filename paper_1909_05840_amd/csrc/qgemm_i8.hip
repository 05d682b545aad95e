// Forward of the group-quantized linear layer on the gfx950 int8 matrix cores.
//
//   acc[t,n] = sum_j x'[t,j] * b[n,j]       v_mfma_i32_32x32x32_i8, int32 accumulators
//   A4[t,n]  = 4*acc + 2*e*rs_x[t] + 2*rs_w[n] + K
//   Y[t,n]   = (h_x*h_g(n)) * float(A4) (+ bias[n])
//
// b is the int8 the matrix core sees: the unsigned code u itself for 2/3/4 bits (e = -L) and
// u - 128 for 8 bits (e = +1); either way A4 equals sum_j (2x'+1)(2u-L), the integer the
// paper's "integer matmul followed by de-quantization" has to produce.
//
// Data movement.  The token tile of X' is copied global -> LDS by the load unit itself
// (global_load_lds_dwordx4, no registers involved), double buffered, into a dense 128-byte-row
// layout whose 16-byte chunks are XOR-swizzled by the row number so that the MFMA fragment
// reads are free of bank conflicts.  The packed weights never touch LDS: the packed
// layout stores, per 32-neuron block and 64-feature unit, one slot per lane, so a wavefront
// fetches its B operand with one coalesced load and expands the k-bit codes to int8 with a few
// byte-parallel shifts and masks in registers, right in front of the MFMA that consumes them.
// Workgroups are renumbered so that the ones sharing a token panel run on the same XCD (same L2).
#include "qb_common.hpp"

namespace qb {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

template <int BITS, int TM, int TN, int WM, int WN, int KU>
__global__ __launch_bounds__(64 * WM * WN) void qgemm_i8_kernel(
    const int8_t *__restrict__ Xq, const int32_t *__restrict__ rs_x, const uint8_t *__restrict__ packed,
    const float *__restrict__ h, const int32_t *__restrict__ rs_w, const float *__restrict__ bias,
    float *__restrict__ Y, int32_t *__restrict__ A4out, int T, int N, int K, int rows_per_group, float hx,
    int tiles_m, int tiles_n)
{
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
        const int bid = blockIdx.x, xcd = bid & 7, idx = bid >> 3;
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
        const float scale = hx * h[nn / rows_per_group];
        const float bv = bias ? bias[nn] : 0.0f;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int t0 = tile_m * BM + (wm * TM + tm) * 32 + 4 * hf;
            if (interior) {
                int rx[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) rx[i] = rs_x[t0 + 8 * (i >> 2) + (i & 3)];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = t0 + 8 * (i >> 2) + (i & 3);
                    const int a4 = 4 * acc[tm][tn][i] + E2 * rx[i] + coln;
                    const size_t at = (size_t)t * N + n;
                    Y[at] = scale * (float)a4 + bv;
                    if (A4out) A4out[at] = a4;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = t0 + 8 * (i >> 2) + (i & 3);
                    if (t < T && n_ok) {
                        const int a4 = 4 * acc[tm][tn][i] + E2 * rs_x[t] + coln;
                        const size_t at = (size_t)t * N + n;
                        Y[at] = scale * (float)a4 + bv;
                        if (A4out) A4out[at] = a4;
                    }
                }
            }
        }
    }
}

#define QB_GLOBAL_TO_LDS16(gptr, lptr)                                                                   \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gptr),             \
                                     (__attribute__((address_space(3))) void *)(lptr), 16, 0, 0)

// Main kernel, K a multiple of 128.  One K-step is 128 features: two 64-code units per lane.
template <int BITS, int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN) void qgemm_i8_dma_kernel(
    const int8_t *__restrict__ Xq, const int32_t *__restrict__ rs_x, const uint8_t *__restrict__ packed,
    const float *__restrict__ h, const int32_t *__restrict__ rs_w, const float *__restrict__ bias,
    float *__restrict__ Y, int32_t *__restrict__ A4out, int T, int N, int K, int rows_per_group, float hx,
    int tiles_m, int tiles_n)
{
    constexpr int NW = WM * WN;
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 128;
    constexpr int DMA_PER_WAVE = BM / 8 / NW;  // each DMA instruction of a wave fills 8 rows of 128 bytes
    static_assert(BM % (8 * NW) == 0, "token tile must split into 8-row blocks per wavefront");
    constexpr int SLOT = 4 * BITS;

    // two separate objects: accesses to one are known not to alias the copy in flight to the other
    __shared__ __align__(1024) uint8_t lds0[BM * BK];
    __shared__ __align__(1024) uint8_t lds1[BM * BK];

    const int nwg = tiles_m * tiles_n;
    int logical;
    {
        const int bid = blockIdx.x, xcd = bid & 7, idx = bid >> 3;
        const int q = nwg >> 3, r = nwg & 7;
        logical = xcd * q + (xcd < r ? xcd : r) + idx;
    }
    const int tile_m = logical / tiles_n, tile_n = logical - tile_m * tiles_n;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave - wm * WN;
    const int l32 = lane & 31, hf = lane >> 5;

    // ---- token tile: lane l of a DMA instruction fills physical chunk l%8 of row l/8 of an 8-row
    // block, which holds logical chunk (l%8) ^ (row%8)
    const int8_t *a_base = Xq + (size_t)tile_m * BM * K;
    const int last_row = T - 1 - tile_m * BM;  // rows past the end re-read the last one; outputs masked
    uint32_t a_off[DMA_PER_WAVE];
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; ++i) {
        int row = (i * NW + wave) * 8 + (lane >> 3);
        row = row < last_row ? row : last_row;
        a_off[i] = (uint32_t)row * (uint32_t)K + (uint32_t)(((lane & 7) ^ (lane >> 3)) * 16);
    }
    // fragment reads: row = wm*TM*32 + tm*32 + l32, logical chunk = kk*4 + hf*2 + sub
    const int p0 = (hf * 2) ^ (l32 & 7);
    const int frag_row = (wm * TM * 32 + l32) * BK;
    int a_frag[4];
    a_frag[0] = frag_row + ((p0 ^ 0) << 4);  // kk 0, sub 0
    a_frag[1] = frag_row + ((p0 ^ 1) << 4);  // kk 0, sub 1
    a_frag[2] = frag_row + ((p0 ^ 4) << 4);  // kk 1, sub 0
    a_frag[3] = frag_row + ((p0 ^ 5) << 4);  // kk 1, sub 1

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

    uint32_t b0[TN][2][BITS], b1[TN][2][BITS];

#define QB_FETCH(step, BDST, LDSDST)                                                                      \
    {                                                                                                     \
        _Pragma("unroll") for (int tn = 0; tn < TN; ++tn)                                                 \
            _Pragma("unroll") for (int kk = 0; kk < 2; ++kk) {                                            \
                const uint32_t *p_ =                                                                      \
                    reinterpret_cast<const uint32_t *>(b_src[tn] + (size_t)((step) * 2 + kk) * 64 * SLOT); \
                _Pragma("unroll") for (int i = 0; i < BITS; ++i) BDST[tn][kk][i] = p_[i];                 \
            }                                                                                             \
        _Pragma("unroll") for (int i = 0; i < DMA_PER_WAVE; ++i)                                          \
            QB_GLOBAL_TO_LDS16(a_base + a_off[i] + (size_t)(step) * BK, LDSDST + (i * NW + wave) * 1024); \
        __builtin_amdgcn_sched_barrier(0); /* fetches stay ahead of the MFMAs that hide their latency */ \
    }
#define QB_MMA(LDSSRC, BSRC)                                                                              \
    {                                                                                                     \
        _Pragma("unroll") for (int kk = 0; kk < 2; ++kk) {                                                \
            uint32_t d[TN][8];                                                                            \
            _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) {                                           \
                unpack_run<BITS>(BSRC[tn][kk], d[tn]);                                                    \
                if constexpr (BITS == 8) {                                                                \
                    _Pragma("unroll") for (int i = 0; i < 8; ++i) d[tn][i] ^= 0x80808080u;                \
                }                                                                                         \
            }                                                                                             \
            _Pragma("unroll") for (int sub = 0; sub < 2; ++sub) {                                         \
                v4i a[TM], b[TN];                                                                         \
                _Pragma("unroll") for (int tm = 0; tm < TM; ++tm) a[tm] =                                 \
                    *reinterpret_cast<const v4i *>(LDSSRC + a_frag[kk * 2 + sub] + tm * 32 * BK);         \
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
// all copies issued so far have landed (vmcnt = 0), then let every wavefront see them
#define QB_JOIN()                                                                                         \
    {                                                                                                     \
        __builtin_amdgcn_s_waitcnt(0x0F70);                                                               \
        __syncthreads();                                                                                  \
    }

    const int nsteps = K / BK;
    QB_FETCH(0, b0, lds0)
    QB_JOIN()
    int s = 0;
    for (; s + 2 < nsteps; s += 2) {
        QB_FETCH(s + 1, b1, lds1)
        QB_MMA(lds0, b0)
        QB_JOIN()
        QB_FETCH(s + 2, b0, lds0)
        QB_MMA(lds1, b1)
        QB_JOIN()
    }
    if (nsteps - s == 2) {
        QB_FETCH(s + 1, b1, lds1)
        QB_MMA(lds0, b0)
        QB_JOIN()
        QB_MMA(lds1, b1)
    } else {
        QB_MMA(lds0, b0)
    }
#undef QB_FETCH
#undef QB_MMA
#undef QB_JOIN

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
        const float scale = hx * h[nn / rows_per_group];
        const float bv = bias ? bias[nn] : 0.0f;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int t0 = tile_m * BM + (wm * TM + tm) * 32 + 4 * hf;
            if (interior) {
                int rx[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) rx[i] = rs_x[t0 + 8 * (i >> 2) + (i & 3)];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = t0 + 8 * (i >> 2) + (i & 3);
                    const int a4 = 4 * acc[tm][tn][i] + E2 * rx[i] + coln;
                    const size_t at = (size_t)t * N + n;
                    Y[at] = scale * (float)a4 + bv;
                    if (A4out) A4out[at] = a4;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = t0 + 8 * (i >> 2) + (i & 3);
                    if (t < T && n_ok) {
                        const int a4 = 4 * acc[tm][tn][i] + E2 * rs_x[t] + coln;
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
void launch_cfg(const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
                const float *bias, float *Y, int32_t *A4, int T, int N, int K, int rpg, float hx, hipStream_t st)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL((qgemm_i8_kernel<BITS, TM, TN, WM, WN, KU>), dim3(tiles_m * tiles_n), dim3(64 * WM * WN), 0, st,
                       Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, tiles_m, tiles_n);
}

template <int BITS, int TM, int TN, int WM, int WN>
void launch_dma(const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
                const float *bias, float *Y, int32_t *A4, int T, int N, int K, int rpg, float hx, hipStream_t st)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    const int tiles_m = (T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL((qgemm_i8_dma_kernel<BITS, TM, TN, WM, WN>), dim3(tiles_m * tiles_n), dim3(64 * WM * WN), 0, st,
                       Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, tiles_m, tiles_n);
}

template <int BITS>
void launch_bits(const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
                 const float *bias, float *Y, int32_t *A4, int T, int N, int K, int rpg, float hx, hipStream_t st)
{
    if (K % 128 != 0) {  // odd number of 64-feature units: register-staged kernel, one unit per step
        launch_cfg<BITS, 2, 2, 2, 2, 1>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st);
        return;
    }
    const long big_tiles = (long)((T + 255) / 256) * ((N + 127) / 128);
    if (big_tiles >= 192) launch_dma<BITS, 4, 2, 2, 2>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st);
    else launch_dma<BITS, 2, 2, 2, 2>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st);
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
