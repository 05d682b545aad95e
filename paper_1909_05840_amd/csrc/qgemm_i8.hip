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
// Data movement.  The token tile of X' goes global -> registers -> LDS (double buffered) and
// is shared by the wavefronts of a workgroup.  The packed weights never touch LDS: the packed
// layout stores, per 32-neuron block and 64-feature unit, one slot per lane, so a wavefront
// fetches its B operand with one coalesced load and expands the k-bit codes to int8 with a few
// byte-parallel shifts and masks in registers, right in front of the MFMA that consumes them.
// Workgroups are renumbered so that the ones sharing a token panel run on the same XCD (same L2).
#include "qb_common.hpp"

namespace qb {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

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

    uint4 areg[A_PER_THREAD];
    uint32_t breg[TN][KU][BITS];

    auto load_global = [&](int step) {
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i)
            areg[i] = *reinterpret_cast<const uint4 *>(a_src[i] + (size_t)step * BK);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int kk = 0; kk < KU; ++kk) {
                const uint32_t *p =
                    reinterpret_cast<const uint32_t *>(b_src[tn] + (size_t)(step * KU + kk) * 64 * SLOT);
#pragma unroll
                for (int i = 0; i < BITS; ++i) breg[tn][kk][i] = p[i];
            }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) *reinterpret_cast<uint4 *>(&lds[buf][a_dst[i]]) = areg[i];
    };

    const int nsteps = K / BK;
    load_global(0);
    store_lds(0);
    uint32_t bcur[TN][KU][BITS];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int kk = 0; kk < KU; ++kk)
#pragma unroll
            for (int i = 0; i < BITS; ++i) bcur[tn][kk][i] = breg[tn][kk][i];
    __syncthreads();

    const int a_frag_base = (wm * TM * 32 + l32) * LDA + hf * 32;

    for (int s = 0; s < nsteps; ++s) {
        if (s + 1 < nsteps) load_global(s + 1);
        const uint8_t *abuf = lds[s & 1];
#pragma unroll
        for (int kk = 0; kk < KU; ++kk) {
            uint32_t d[TN][8];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                unpack_run<BITS>(bcur[tn][kk], d[tn]);
                if constexpr (BITS == 8) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) d[tn][i] ^= 0x80808080u;
                }
            }
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                v4i a[TM], b[TN];
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    a[tm] = *reinterpret_cast<const v4i *>(abuf + a_frag_base + tm * 32 * LDA + kk * 64 + sub * 16);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    b[tn][0] = (int)d[tn][4 * sub + 0];
                    b[tn][1] = (int)d[tn][4 * sub + 1];
                    b[tn][2] = (int)d[tn][4 * sub + 2];
                    b[tn][3] = (int)d[tn][4 * sub + 3];
                }
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
            }
        }
        if (s + 1 < nsteps) {
            store_lds((s + 1) & 1);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int kk = 0; kk < KU; ++kk)
#pragma unroll
                    for (int i = 0; i < BITS; ++i) bcur[tn][kk][i] = breg[tn][kk][i];
        }
        __syncthreads();
    }

    // ---- epilogue: exact integer corrections, then one scale per column
    constexpr int L = (1 << BITS) - 1;
    constexpr int E2 = (BITS == 8) ? 2 : -2 * L;  // 2*e
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
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int t = t0 + 8 * (i >> 2) + (i & 3);
                if (t < T && n_ok) {
                    const int a4 = 4 * acc[tm][tn][i] + E2 * rs_x[t] + coln;
                    const size_t at = (size_t)t * N + n;
                    float y = scale * (float)a4;
                    if (bias) y += bv;
                    Y[at] = y;
                    if (A4out) A4out[at] = a4;
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

template <int BITS>
void launch_bits(const int8_t *Xq, const int32_t *rs_x, const uint8_t *packed, const float *h, const int32_t *rs_w,
                 const float *bias, float *Y, int32_t *A4, int T, int N, int K, int rpg, float hx, hipStream_t st)
{
    const bool k128 = (K % 128) == 0;
    const long big_tiles = (long)((T + 255) / 256) * ((N + 127) / 128);
    if (big_tiles >= 192) {
        if (k128) launch_cfg<BITS, 4, 2, 2, 2, 2>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st);
        else launch_cfg<BITS, 4, 2, 2, 2, 1>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st);
    } else {
        if (k128) launch_cfg<BITS, 2, 2, 2, 2, 2>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st);
        else launch_cfg<BITS, 2, 2, 2, 2, 1>(Xq, rs_x, packed, h, rs_w, bias, Y, A4, T, N, K, rpg, hx, st);
    }
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
