// Straight-through backward of the group-quantized linear layer on the gfx950 bf16 matrix
// cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
//   dX[t,j] = sum_n dY[t,n] * What[n,j]     What[n,j] = h_g(n) * (2u[n,j] - L)
//   dW[n,j] = sum_t dY[t,n] * Xhat[t,j]     Xhat[t,j] = h_x * (2x'[t,j] + 1)
//
// Both products are brought to the form C[M,Nc] = sum_k A[M,k] * B[Nc,k] (both operands
// contiguous along the contraction) by staging operands in the caller's workspace:
//   WT  [K, Np]   bf16(What) transposed, Np = N rounded up to 64, zero padded
//   dYp [T, Np]   dY zero padded along n (only when N is not a multiple of 64)
//   dYT [N, Tp]   dY transposed, Tp = T rounded up to 64, zero padded
//   XT  [K, Tp]   (2x'+1) transposed; |2x'+1| <= 255 is exact in bf16, h_x goes to the epilogue
// dW splits the long contraction over T across workgroups; partial sums are written to the
// workspace and added in a fixed order, so results do not change from run to run.
#include "qb_common.hpp"
#include <mutex>

namespace qb {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x)
{
    uint32_t b = __float_as_uint(x);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}

inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

// packed slots -> WT[j][n] = bf16(h_g * (2u - L)), or with asymmetric ranges (q0 given, h holds Delta)
// bf16(Delta_g * u + q0_g); one thread per (n, 32-code run); n < Np
template <int BITS>
__device__ __forceinline__ void dequant_transpose_body(int bx, const uint8_t *__restrict__ packed,
                                                       const float *__restrict__ h, const float *__restrict__ q0, int N,
                                                       int Np, int K, int rows_per_group, uint16_t *__restrict__ WT)
{
    const int runs = K >> 5;
    const int64_t id = (int64_t)bx * 256 + threadIdx.x;
    if (id >= (int64_t)Np * runs) return;
    const int rc = (int)(id / Np), n = (int)(id % Np);  // consecutive threads: consecutive n
    uint16_t *dst = WT + (size_t)(rc * 32) * Np + n;
    if (n >= N) {
#pragma unroll
        for (int i = 0; i < 32; ++i) dst[(size_t)i * Np] = 0;
        return;
    }
    const uint32_t *src = reinterpret_cast<const uint32_t *>(packed + slot_index(n, rc, K) * (size_t)(4 * BITS));
    uint32_t in[BITS], d[8];
#pragma unroll
    for (int i = 0; i < BITS; ++i) in[i] = src[i];
    unpack_run<BITS>(in, d);
    const float hg = h[n / rows_per_group];
    constexpr int L = (1 << BITS) - 1;
    if (q0) {
        const float z = q0[n / rows_per_group];
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const int u = (int)((d[i >> 2] >> (8 * (i & 3))) & 255u);
            dst[(size_t)i * Np] = f32_to_bf16_rne(hg * (float)u + z);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const int u = (int)((d[i >> 2] >> (8 * (i & 3))) & 255u);
        dst[(size_t)i * Np] = f32_to_bf16_rne(hg * (float)(2 * u - L));
    }
}

// out[c][r] = conv(in[r][c]) for r < R, c < C; out has leading dimension ldo >= R (a multiple of 64),
// columns r in [R, ldo) are zero filled.  MODE 0: bf16 copy, MODE 1: int8 x' -> bf16(2x'+1).
// A block moves a 64x64 tile through LDS: rows are read with 16-byte (MODE 0) or 8-byte (MODE 1)
// loads when C allows it, and every thread writes 8 consecutive r of one output row with one
// 16-byte store.
template <int MODE>
__device__ __forceinline__ void transpose_body(int bx, int by, uint16_t (*tile)[66], const void *__restrict__ in, int R,
                                               int C, int ldo, uint16_t *__restrict__ out)
{
    const int r0 = bx * 64, c0 = by * 64;
    const int tid = threadIdx.x;
    const bool vec = (C % 8 == 0);  // uniform: rows are then 16-byte (MODE 0) / 8-byte (MODE 1) aligned
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int i = (tid >> 3) + it * 32;  // row of the tile
        const int j = (tid & 7) * 8;         // first of 8 columns
        const int r = r0 + i, c = c0 + j;
        uint16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = 0;
        if (r < R) {
            if (vec && c + 8 <= C) {
                if (MODE == 0) {
                    const uint4 q = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(in) + (size_t)r * C + c);
                    v[0] = q.x & 0xFFFF; v[1] = q.x >> 16; v[2] = q.y & 0xFFFF; v[3] = q.y >> 16;
                    v[4] = q.z & 0xFFFF; v[5] = q.z >> 16; v[6] = q.w & 0xFFFF; v[7] = q.w >> 16;
                } else {
                    const uint2 q = *reinterpret_cast<const uint2 *>(static_cast<const int8_t *>(in) + (size_t)r * C + c);
                    const uint32_t w[2] = {q.x, q.y};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int x = (int)(int8_t)((w[e >> 2] >> (8 * (e & 3))) & 0xFF);
                        v[e] = (uint16_t)(__float_as_uint((float)(2 * x + 1)) >> 16);  // exact: 8 significant bits
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (c + e < C) {
                        if (MODE == 0) {
                            v[e] = static_cast<const uint16_t *>(in)[(size_t)r * C + c + e];
                        } else {
                            const int x = static_cast<const int8_t *>(in)[(size_t)r * C + c + e];
                            v[e] = (uint16_t)(__float_as_uint((float)(2 * x + 1)) >> 16);
                        }
                    }
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) tile[i][j + e] = v[e];
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int c = (tid >> 3) + it * 32;  // output row inside the tile
        const int rr = (tid & 7) * 8;        // first of 8 consecutive r
        if (c0 + c < C) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (uint32_t)tile[rr + 2 * e][c] | ((uint32_t)tile[rr + 2 * e + 1][c] << 16);
            *reinterpret_cast<uint4 *>(out + (size_t)(c0 + c) * ldo + r0 + rr) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

// The operands of both backward GEMMs staged by one launch: blocks [0, nb_w) de-quantize and transpose the weights
// (for dX), the next nb_y blocks transpose dY and the last nb_x blocks transpose-and-convert the activation codes
// (for dW).  A section with zero blocks is skipped.
struct StageArgs {
    const uint8_t *packed; const float *h; const float *q0; int N, Np, K, rows_per_group; uint16_t *WT; int nb_w;
    const uint16_t *dY; int T, Tp; uint16_t *dYT; int nb_y;
    const int8_t *Xq; uint16_t *XT; int nb_x;
};

template <int BITS>
__global__ __launch_bounds__(256) void stage_operands_kernel(const StageArgs a)
{
    __shared__ uint16_t tile[64][66];
    int b = blockIdx.x;
    if (b < a.nb_w) {
        dequant_transpose_body<BITS>(b, a.packed, a.h, a.q0, a.N, a.Np, a.K, a.rows_per_group, a.WT);
        return;
    }
    b -= a.nb_w;
    const int tb = a.Tp / 64;  // tiles along T
    if (b < a.nb_y) {
        transpose_body<0>(b % tb, b / tb, tile, a.dY, a.T, a.N, a.Tp, a.dYT);
        return;
    }
    b -= a.nb_y;
    transpose_body<1>(b % tb, b / tb, tile, a.Xq, a.T, a.K, a.Tp, a.XT);
}

// dYp[t][n] = dY[t][n] for n < N, 0 for N <= n < Np
__global__ __launch_bounds__(256) void pad_rows_kernel(const uint16_t *__restrict__ in, int64_t T, int N, int Np,
                                                       uint16_t *__restrict__ out)
{
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= T * Np) return;
    const int64_t t = id / Np;
    const int n = (int)(id % Np);
    out[id] = n < N ? in[t * N + n] : (uint16_t)0;
}

// global -> LDS copy by the load unit (every lane its own global address; lane l lands at m0 + 16*l).
// Inline assembly on purpose: the kernel states itself, with s_waitcnt vmcnt(n), which copies must have
// landed before a barrier.
__device__ __forceinline__ void copy16_to_lds(const void *g, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0070 | 0x0F00);
}

// C[M,Nc] = sum_k A[M,k] * B[Nc,k]; A, B bf16 row-major with leading dimensions lda, ldb
// (multiples of 8), contraction range [z*ksplit, min(Kc, (z+1)*ksplit)) for blockIdx.y = z,
// Kc and ksplit multiples of 64.  OUT 0: bf16 C (ldc = Nc);  OUT 1: fp32 C * scale;
// OUT 2: fp32 partial sums at part + z*M*Nc.
// Both operand tiles (64 bf16 = 128 bytes per row and step) are copied global -> LDS by the load
// unit through a ring of NSTAGE stages; rows are dense with their 16-byte chunks XOR-swizzled by
// (row/2)%8, so the 16-byte MFMA fragment reads are free of bank conflicts.  The grid is persistent
// over the tiles of one contraction split and renumbered per XCD like the forward kernel.
// The work is split by role and by SIMD.  The wavefronts of a workgroup are dealt to the
// four SIMDs of the CU in turn (wavefront w on SIMD w%4), and a global -> LDS copy issued on a SIMD that is
// busy with 32x32 MFMAs runs at about half speed (and slows the MFMAs), while one issued on a SIMD without
// MFMAs does not.  Hence: wavefronts 3 and 7 (SIMD 3) do nothing but copy, wavefronts 0,1,2,4,5,6 multiply,
// 64 x 32 outputs each in a 2 x 3 grid: tiles of 128 x 96.  Per step and tile, 28 KB are copied for 522
// cycles of MFMAs on each of three SIMDs.  (Roles depend on the wavefront number only: a different
// placement by the hardware would cost speed, not correctness.)
// Protocol per tile (n steps, ring of NSTAGE stages, copies run D = NSTAGE-1 steps ahead); every wavefront
// executes n+1 barriers:
//   copy wavefronts: start copies 0..D-1; wait copy 0; BARRIER;
//                    for s: start copy s+D (its stage was read in step s-1, finished at the last barrier);
//                           wait copy s+1 (vmcnt leaves the younger ones in flight); BARRIER
//   MFMA wavefronts: BARRIER; for s: multiply stage s % NSTAGE; BARRIER
// The clamp's derivative (MASK): element (r, n) of the result is set to zero where |src[r, n]| exceeds its
// range: lim[r / rows_per_lim] for dW (weights: one range per group of rows), lim_all for dX.
struct ClampMask {
    const float *src;
    const float *lim;
    float lim_all;
    int rows_per_lim;
};

template <int NSTAGE, int OUT, bool MASK, int TM>
__global__ __launch_bounds__(512) void gemm_bf16_nt_s3_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, int M, int Nc, int Kc, int lda, int ldb,
    int ksplit, float scale, void *__restrict__ Cout, int tiles_m, int tiles_n, const ClampMask mask)
{
    // TM 32-row blocks per MFMA wavefront: tiles of 64*TM x 96 (128 x 96, or 256 x 96 where that still fills the chip:
    // half as many tile changes, a weight fragment serves four MFMAs instead of two)
    constexpr int WN = 3, NPROD = 2;
    constexpr int BM = 64 * TM, BN = 96, BKB = 128;  // 64 bf16 per step
    constexpr int A_TOTAL = BM / 8, B_TOTAL = BN / 8;
    constexpr int A_PER = A_TOTAL / NPROD, B_PER = B_TOTAL / NPROD, PERP = A_PER + B_PER;
    constexpr int D = NSTAGE - 1;
    constexpr int A_BYTES = BM * BKB, STAGE_BYTES = (BM + BN) * BKB;
    static_assert((D - 1) * PERP < 64, "vmcnt has six bits");
    __shared__ __align__(1024) uint8_t lds[NSTAGE * STAGE_BYTES];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int z = blockIdx.y;
    const int k_begin = z * ksplit;
    const int k_end = (k_begin + ksplit < Kc) ? k_begin + ksplit : Kc;
    const int nsteps = (k_end - k_begin) >> 6;
    const int nwg = tiles_m * tiles_n;
    auto tile_of = [&](int work, int &tile_m, int &tile_n) {
        const int xcd = work & 7, idx = work >> 3;
        const int q = nwg >> 3, r = nwg & 7;
        const int logical = xcd * q + (xcd < r ? xcd : r) + idx;
        tile_m = logical / tiles_n;
        tile_n = logical - tile_m * tiles_n;
    };

    if ((wave & 3) == 3) {
        // ================================ copies ================================
        const int p = wave >> 2;
        for (int work = blockIdx.x; work < nwg; work += gridDim.x) {
            int tile_m, tile_n;
            tile_of(work, tile_m, tile_n);
            const uint8_t *a_src[A_PER], *b_src[B_PER];
            uint32_t a_dst[A_PER], b_dst[B_PER];
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                const int blk = i * NPROD + p;
                const int row = blk * 8 + (lane >> 3);
                const int kx = (row >> 1) & 7;
                int r = tile_m * BM + row;
                r = r < M ? r : M - 1;  // rows past the end re-read the last one; outputs masked
                a_src[i] = reinterpret_cast<const uint8_t *>(A + (size_t)r * lda + k_begin) + (((lane & 7) ^ kx) * 16);
                a_dst[i] = blk * 1024;
            }
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int blk = i * NPROD + p;
                const int row = blk * 8 + (lane >> 3);
                const int kx = (row >> 1) & 7;
                int r = tile_n * BN + row;
                r = r < Nc ? r : Nc - 1;
                b_src[i] = reinterpret_cast<const uint8_t *>(B + (size_t)r * ldb + k_begin) + (((lane & 7) ^ kx) * 16);
                b_dst[i] = A_BYTES + blk * 1024;
            }
            auto fetch = [&](int step, int stage) {
                const uint32_t st_ = lds_base + stage * STAGE_BYTES;
#pragma unroll
                for (int i = 0; i < A_PER; ++i) copy16_to_lds(a_src[i] + (size_t)step * BKB, st_ + a_dst[i]);
#pragma unroll
                for (int i = 0; i < B_PER; ++i) copy16_to_lds(b_src[i] + (size_t)step * BKB, st_ + b_dst[i]);
            };
#pragma unroll
            for (int u = 0; u < D; ++u)
                if (u < nsteps) fetch(u, u);
            if (nsteps >= D) wait_vmcnt<(D - 1) * PERP>();
            else wait_vmcnt<0>();
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
        return;
    }

    // ================================ MFMA ================================
    const int cidx = (wave & 3) + 3 * (wave >> 2);
    const int wm = cidx / WN, wn = cidx - wm * WN;
    const int l32 = lane & 31, hf = lane >> 5;
    // fragment reads: row r, logical chunk = sub*2 + hf, physical chunk = logical ^ ((r/2)%8)
    const int key = (l32 >> 1) & 7;
    int a_frag[4], b_frag[4];
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
        a_frag[sub] = (wm * TM * 32 + l32) * BKB + (((sub * 2 + hf) ^ key) << 4);
        b_frag[sub] = A_BYTES + (wn * 32 + l32) * BKB + (((sub * 2 + hf) ^ key) << 4);
    }
    for (int work = blockIdx.x; work < nwg; work += gridDim.x) {
        int tile_m, tile_n;
        tile_of(work, tile_m, tile_n);
        v16f acc[TM];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tm][i] = 0.0f;
        // The clamp mask's source values for this wavefront's 64 x 32 results, loaded before the K-loop (which hides
        // their latency) as 2 x 4 float4: one instruction covers 8 rows x 32 columns, lane l the row l/8 and the four
        // columns 4*(l%8)... of it.  That is not the accumulator's lane layout: after the K-loop every lane turns its
        // values into predicate bits, and the bits change lanes (below).  Rows and columns past the end re-read valid
        // elements; their results are not stored.  No load may be left for the write-out: waiting for it there would
        // also wait for every store before it.
        float4 mv[TM][4];
        float ml[TM][4];
        if constexpr (MASK && OUT != 2) {
            int cc = tile_n * BN + wn * 32 + 4 * (lane & 7);
            cc = cc < Nc ? cc : Nc - 4;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    int r = tile_m * BM + (wm * TM + tm) * 32 + 8 * q + (lane >> 3);
                    r = r < M ? r : M - 1;
                    mv[tm][q] = *reinterpret_cast<const float4 *>(mask.src + (size_t)r * Nc + cc);
                    ml[tm][q] = (OUT == 1) ? mask.lim[r / mask.rows_per_lim] : mask.lim_all;
                }
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        int stage = 0;
        for (int s = 0; s < nsteps; ++s) {
            const uint8_t *st_ = lds + stage * STAGE_BYTES;
            v8bf af[4][TM], bf[4];
#pragma unroll
            for (int sub = 0; sub < 4; ++sub) {
                bf[sub] = *reinterpret_cast<const v8bf *>(st_ + b_frag[sub]);
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) af[sub][tm] = *reinterpret_cast<const v8bf *>(st_ + a_frag[sub] + tm * 32 * BKB);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int sub = 0; sub < 4; ++sub)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    acc[tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[sub][tm], bf[sub], acc[tm], 0, 0, 0);
            stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        // All mask decisions first, as one bit each, so that the stores below depend on no load.  A lane packs the
        // predicates of its 4 x 4 loaded values into 16 bits (nibble q = load q); the lane that holds the result of
        // row 4*hf + 8*q + j, column l32 finds them in lane (4*hf + j)*8 + l32/4, bit 4*q + l32%4.
        uint64_t outside = 0;
        if constexpr (MASK && OUT != 2) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                uint32_t w = 0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    // the empty statement consumes the loaded values here, so the compiler places its waits for
                    // the loads here and not next to uses it would otherwise sink between the stores
                    asm volatile("" : "+v"(mv[tm][q].x), "+v"(mv[tm][q].y), "+v"(mv[tm][q].z), "+v"(mv[tm][q].w), "+v"(ml[tm][q]));
                    const float lim = ml[tm][q];
                    w |= (fabsf(mv[tm][q].x) > lim ? 1u : 0u) << (4 * q);
                    w |= (fabsf(mv[tm][q].y) > lim ? 2u : 0u) << (4 * q);
                    w |= (fabsf(mv[tm][q].z) > lim ? 4u : 0u) << (4 * q);
                    w |= (fabsf(mv[tm][q].w) > lim ? 8u : 0u) << (4 * q);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t g = (uint32_t)__shfl((int)w, (4 * hf + j) * 8 + (l32 >> 2)) >> (l32 & 3);
#pragma unroll
                    for (int q = 0; q < 4; ++q) outside |= (uint64_t)((g >> (4 * q)) & 1u) << (tm * 16 + 4 * q + j);
                }
            }
            // applied here, as selects: inside the bounds-checked store loop the compiler turns the same test into
            // a branch per element (seventy instructions per store instead of eleven, 4 us per tile)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tm][i] = ((outside >> (tm * 16 + i)) & 1ull) ? 0.0f : acc[tm][i];
        }
        const int n = tile_n * BN + wn * 32 + l32;
        const bool interior = (tile_m + 1) * BM <= M && (tile_n + 1) * BN <= Nc;  // uniform over the workgroup
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int r0 = tile_m * BM + (wm * TM + tm) * 32 + 4 * hf;
            if (interior) {  // no per-element checks, one base address per block
                const size_t at0 = (size_t)r0 * Nc + n + (OUT == 2 ? (size_t)z * M * Nc : 0);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const size_t at = at0 + (size_t)(8 * (i >> 2) + (i & 3)) * Nc;
                    // results that no kernel of this call reads again are streamed past the caches
                    if (OUT == 0) __builtin_nontemporal_store(f32_to_bf16_rne(acc[tm][i]), static_cast<uint16_t *>(Cout) + at);
                    else if (OUT == 1) __builtin_nontemporal_store(acc[tm][i] * scale, static_cast<float *>(Cout) + at);
                    else static_cast<float *>(Cout)[at] = acc[tm][i];
                }
                continue;
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int r = r0 + 8 * (i >> 2) + (i & 3);
                if (r < M && n < Nc) {
                    const size_t at = (size_t)r * Nc + n;
                    if (OUT == 0) static_cast<uint16_t *>(Cout)[at] = f32_to_bf16_rne(acc[tm][i]);
                    else if (OUT == 1) static_cast<float *>(Cout)[at] = acc[tm][i] * scale;
                    else static_cast<float *>(Cout)[(size_t)z * M * Nc + at] = acc[tm][i];
                }
            }
        }
    }
}

// out[row, 4c..4c+3] = scale * sum_z part[z][row, 4c..4c+3]; grid (ceil(cols/1024), rows)
template <bool MASK>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float4 *__restrict__ part, int rows, int cols,
                                                              int splits, float scale, float4 *__restrict__ out,
                                                              const ClampMask mask)
{
    const int c4 = blockIdx.x * 256 + threadIdx.x, row = blockIdx.y;
    if (c4 >= (cols >> 2)) return;
    const size_t at = (size_t)row * (cols >> 2) + c4, n4 = (size_t)rows * (cols >> 2);
    float4 s = part[at];
    for (int z = 1; z < splits; ++z) {
        const float4 v = part[(size_t)z * n4 + at];
        s.x += v.x;
        s.y += v.y;
        s.z += v.z;
        s.w += v.w;
    }
    if constexpr (MASK) {
        const float lim = mask.lim[row / mask.rows_per_lim];
        const float4 w = reinterpret_cast<const float4 *>(mask.src)[at];
        if (fabsf(w.x) > lim) s.x = 0.0f;
        if (fabsf(w.y) > lim) s.y = 0.0f;
        if (fabsf(w.z) > lim) s.z = 0.0f;
        if (fabsf(w.w) > lim) s.w = 0.0f;
    }
    out[at] = make_float4(s.x * scale, s.y * scale, s.z * scale, s.w * scale);
}

template <int OUT, int TM>
void launch_gemm_tm(const uint16_t *A, const uint16_t *B, int M, int Nc, int Kc, int lda, int ldb, int splits, int ksplit,
                    float scale, void *C, hipStream_t st, const ClampMask *mask)
{
    // 64*TM x 96 tiles, 3 stages, one workgroup per CU; persistent grid of at most 256 per split
    const int tm = (M + 64 * TM - 1) / (64 * TM), tn = (Nc + 95) / 96;
    int grid = tm * tn;
    if (grid > 256) grid = 256;
    if (mask && OUT != 2)
        hipLaunchKernelGGL((gemm_bf16_nt_s3_kernel<3, OUT, true, TM>), dim3(grid, splits), dim3(512), 0, st, A, B, M, Nc, Kc,
                           lda, ldb, ksplit, scale, C, tm, tn, *mask);
    else
        hipLaunchKernelGGL((gemm_bf16_nt_s3_kernel<3, OUT, false, TM>), dim3(grid, splits), dim3(512), 0, st, A, B, M, Nc, Kc,
                           lda, ldb, ksplit, scale, C, tm, tn, ClampMask{nullptr, nullptr, 0.0f, 1});
}

template <int OUT>
void launch_gemm(const uint16_t *A, const uint16_t *B, int M, int Nc, int Kc, int lda, int ldb, int splits, int ksplit,
                 float scale, void *C, hipStream_t st, const ClampMask *mask = nullptr)
{
    // 256-row tiles where they come out in whole rounds over the 256 CUs, at least two of them
    const long tiles256 = (long)((M + 255) / 256) * ((Nc + 95) / 96);
    if constexpr (OUT != 2) {
        if (splits == 1 && tiles256 >= 512 && tiles256 % 256 == 0) {
            launch_gemm_tm<OUT, 4>(A, B, M, Nc, Kc, lda, ldb, splits, ksplit, scale, C, st, mask);
            return;
        }
    }
    launch_gemm_tm<OUT, 2>(A, B, M, Nc, Kc, lda, ldb, splits, ksplit, scale, C, st, mask);
}

struct BwdPlan {
    int64_t Np, Tp;
    int splits, ksplit;
    size_t off_wt, off_dyp, off_dyt, off_xt, off_part, total;
};

BwdPlan make_plan(int64_t T, int64_t N, int64_t K)
{
    BwdPlan p;
    p.Np = round_up(N, 64);
    p.Tp = round_up(T, 64);
    // split the contraction over T so that at most about 256 workgroups (one per CU) exist, at least
    // 256 rows each
    const int64_t tiles = ((N + 127) / 128) * ((K + 95) / 96);
    int64_t s = 256 / tiles;
    const int64_t max_s = (p.Tp + 255) / 256;
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    p.ksplit = (int)round_up((p.Tp + s - 1) / s, 64);
    p.splits = (int)((p.Tp + p.ksplit - 1) / p.ksplit);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
    p.off_wt = take((size_t)K * p.Np * 2);
    p.off_dyp = take(N % 64 ? (size_t)T * p.Np * 2 : 0);
    p.off_dyt = take((size_t)N * p.Tp * 2);
    p.off_xt = take((size_t)K * p.Tp * 2);
    p.off_part = take(p.splits > 1 ? (size_t)p.splits * N * K * 4 : 0);
    p.total = off;
    return p;
}

}  // namespace
}  // namespace qb

using namespace qb;

extern "C" size_t qb_bwd_workspace_nbytes(int64_t T, int64_t N, int64_t K)
{
    if (T <= 0 || T > (1 << 24) || N <= 0 || N > (1 << 24) || !k_ok(K)) return 0;
    return make_plan(T, N, K).total;
}

static qb_status bwd_ste(const uint16_t *dY, const int8_t *Xq, float clip, const void *packed, const float *h, int bits,
                         int groups, int64_t T, int64_t N, int64_t K, const float *X, const float *W, const float *m,
                         uint16_t *dX, float *dW, void *workspace, void *stream, const float *q0 = nullptr)
{
    if (!dY || !Xq || !packed || !h) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (T <= 0 || T > (1 << 24) || N <= 0 || N > (1 << 24) || !k_ok(K) || groups <= 0 || N % groups != 0)
        return QB_ERR_SHAPE;
    if (!(clip > 0.0f) || !(clip < 3.0e38f)) return QB_ERR_CLIP;
    if (!dX && !dW) return QB_OK;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return QB_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const BwdPlan p = make_plan(T, N, K);
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const int rpg = (int)(N / groups);
    const int Np = (int)p.Np, Tp = (int)p.Tp;

    uint16_t *WT = reinterpret_cast<uint16_t *>(ws + p.off_wt);
    uint16_t *dYT = reinterpret_cast<uint16_t *>(ws + p.off_dyt);
    uint16_t *XT = reinterpret_cast<uint16_t *>(ws + p.off_xt);
    {
        StageArgs a;
        a.packed = static_cast<const uint8_t *>(packed); a.h = h; a.q0 = q0; a.N = (int)N; a.Np = Np; a.K = (int)K; a.rows_per_group = rpg;
        a.WT = WT; a.nb_w = dX ? (int)(((int64_t)Np * (K / 32) + 255) / 256) : 0;
        a.dY = dY; a.T = (int)T; a.Tp = Tp; a.dYT = dYT; a.nb_y = dW ? (Tp / 64) * (int)((N + 63) / 64) : 0;
        a.Xq = Xq; a.XT = XT; a.nb_x = dW ? (Tp / 64) * (int)((K + 63) / 64) : 0;
        const dim3 grid((unsigned)(a.nb_w + a.nb_y + a.nb_x));
        switch (bits) {
            case 2: hipLaunchKernelGGL(stage_operands_kernel<2>, grid, dim3(256), 0, st, a); break;
            case 3: hipLaunchKernelGGL(stage_operands_kernel<3>, grid, dim3(256), 0, st, a); break;
            case 4: hipLaunchKernelGGL(stage_operands_kernel<4>, grid, dim3(256), 0, st, a); break;
            default: hipLaunchKernelGGL(stage_operands_kernel<8>, grid, dim3(256), 0, st, a); break;
        }
    }
    if (dX) {
        const uint16_t *Aop = dY;
        if (N % 64) {
            uint16_t *dYp = reinterpret_cast<uint16_t *>(ws + p.off_dyp);
            hipLaunchKernelGGL(pad_rows_kernel, dim3((unsigned)((T * Np + 255) / 256)), dim3(256), 0, st, dY, T, (int)N, Np, dYp);
            Aop = dYp;
        }
        const ClampMask mx{X, nullptr, clip, 1};
        launch_gemm<0>(Aop, WT, (int)T, (int)K, Np, Np, Np, 1, Np, 1.0f, dX, st, X ? &mx : nullptr);
    }
    if (dW) {
        const float hx = clip / 255.0f;
        const ClampMask mw{W, m, 0.0f, rpg};
        if (p.splits > 1) {
            float *part = reinterpret_cast<float *>(ws + p.off_part);
            const dim3 rgrid((unsigned)((K / 4 + 255) / 256), (unsigned)N);
            launch_gemm<2>(dYT, XT, (int)N, (int)K, Tp, Tp, Tp, p.splits, p.ksplit, 1.0f, part, st);
            const float4 *part4 = reinterpret_cast<const float4 *>(part);
            float4 *dW4 = reinterpret_cast<float4 *>(dW);
            if (W)
                hipLaunchKernelGGL(reduce_partials_kernel<true>, rgrid, dim3(256), 0, st, part4, (int)N, (int)K, p.splits,
                                   hx, dW4, mw);
            else
                hipLaunchKernelGGL(reduce_partials_kernel<false>, rgrid, dim3(256), 0, st, part4, (int)N, (int)K,
                                   p.splits, hx, dW4, mw);
        } else {
            launch_gemm<1>(dYT, XT, (int)N, (int)K, Tp, Tp, Tp, 1, Tp, hx, dW, st, W ? &mw : nullptr);
        }
    }
    return launch_status();
}

extern "C" qb_status qb_qlinear_bwd_ste(const uint16_t *dY, const int8_t *Xq, float clip, const void *packed,
                                        const float *h, int bits, int groups, int64_t T, int64_t N, int64_t K,
                                        uint16_t *dX, float *dW, void *workspace, void *stream)
{
    return bwd_ste(dY, Xq, clip, packed, h, bits, groups, T, N, K, nullptr, nullptr, nullptr, dX, dW, workspace, stream);
}

// ---- the backward for callers that cannot allocate: its staging area is a fixed array of the library -------------
// One array per GPU (every device the code object is loaded on holds its own copy until the process ends).  In host
// code the array's name is not a device address; the address on the current device is asked for once per device
// and kept.
static __device__ __align__(256) unsigned char scratch[QB_BWD_STATIC_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices] = {};

// the current device's copy of `scratch`, or null if the runtime does not give it
void *scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" qb_status qb_qlinear_bwd_ste_static(const uint16_t *dY, const int8_t *Xq, float clip, const void *packed,
                                               const float *h, int bits, int groups, int64_t T, int64_t N, int64_t K,
                                               uint16_t *dX, float *dW, void *stream)
{
    if (T <= 0 || T > (1 << 24) || N <= 0 || N > (1 << 24) || !k_ok(K)) return QB_ERR_SHAPE;
    if (make_plan(T, N, K).total > (size_t)QB_BWD_STATIC_BYTES) return QB_ERR_WORKSPACE;  // larger than the fixed staging area
    void *ws = scratch_of_current_device();
    if (!ws) return QB_ERR_HIP;
    // every byte of the staging area that the GEMMs read is written by this call's own staging launch first
    // (padding included), so the contents a previous call left behind never matter
    return bwd_ste(dY, Xq, clip, packed, h, bits, groups, T, N, K, nullptr, nullptr, nullptr, dX, dW, ws, stream);
}

extern "C" qb_status qb_qlinear_bwd_ste_masked(const uint16_t *dY, const int8_t *Xq, float clip, const void *packed,
                                               const float *h, int bits, int groups, int64_t T, int64_t N, int64_t K,
                                               const float *X, const float *W, const float *m, uint16_t *dX,
                                               float *dW, void *workspace, void *stream)
{
    if ((W == nullptr) != (m == nullptr)) return QB_ERR_NULL;
    return bwd_ste(dY, Xq, clip, packed, h, bits, groups, T, N, K, X, W, m, dX, dW, workspace, stream);
}

extern "C" qb_status qb_qlinear_bwd_ste_asym(const uint16_t *dY, const int8_t *Xq, float clip, const void *packed,
                                             const float *delta, const float *q0, int bits, int groups, int64_t T,
                                             int64_t N, int64_t K, uint16_t *dX, float *dW, void *workspace, void *stream)
{
    if (!q0) return QB_ERR_NULL;
    return bwd_ste(dY, Xq, clip, packed, delta, bits, groups, T, N, K, nullptr, nullptr, nullptr, dX, dW, workspace, stream,
                   q0);
}
