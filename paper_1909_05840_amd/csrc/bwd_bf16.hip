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
// Both products of a call run in one launch whose workgroups share the contraction steps evenly; a tile that two
// or more workgroups worked on has its partial sums added in a fixed order, so results do not change from run
// to run.
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
// (for dW).  A section with zero blocks is skipped.  One last block clears the flags of the GEMM launch.
struct StageArgs {
    const uint8_t *packed; const float *h; const float *q0; int N, Np, K, rows_per_group; uint16_t *WT; int nb_w;
    const uint16_t *dY; int T, Tp; uint16_t *dYT; int nb_y;
    const int8_t *Xq; uint16_t *XT; int nb_x;
    int *flags; int n_flags;  // cleared by one more block (the GEMM launch behind this one raises them)
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
    if (b < a.nb_x) {
        transpose_body<1>(b % tb, b / tb, tile, a.Xq, a.T, a.K, a.Tp, a.XT);
        return;
    }
    for (int i = threadIdx.x; i < a.n_flags; i += 256) a.flags[i] = 0;
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

// C[M,Nc] = sum_k A[M,k] * B[Nc,k]; A, B bf16 row-major with leading dimensions lda, ldb (multiples of 8), the
// contraction length a multiple of 64.  out 0: bf16 C (ldc = Nc); out 1: fp32 C * scale.
// Both operand tiles (64 bf16 = 128 bytes per row and step) are copied global -> LDS by the load
// unit through a ring of NSTAGE stages; rows are dense with their 16-byte chunks XOR-swizzled by
// (row/2)%8, so the 16-byte MFMA fragment reads are free of bank conflicts.
// The work is split by role and by SIMD.  The wavefronts of a workgroup are dealt to the
// four SIMDs of the CU in turn (wavefront w on SIMD w%4), and a global -> LDS copy issued on a SIMD that is
// busy with 32x32 MFMAs runs at about half speed (and slows the MFMAs), while one issued on a SIMD without
// MFMAs does not.  Hence: wavefronts 3 and 7 (SIMD 3) do nothing but copy, wavefronts 0,1,2,4,5,6 multiply,
// in a 2 x 3 grid, 64 x 32 outputs each (tiles of 128 x 96: per step 28 KB copied for 512 cycles of MFMAs on each
// of three SIMDs) or 64 x 64 (tiles of 128 x 192: 40 KB for 1024 cycles).  (Roles depend on the wavefront number
// only: a different placement by the hardware would cost speed, not correctness.)
// Protocol per run of n steps (ring of NSTAGE stages, copies run D = NSTAGE-1 steps ahead); every wavefront
// executes n+1 barriers:
//   copy wavefronts: start copies 0..D-1; wait copy 0; BARRIER;
//                    for s: start copy s+D (its stage was read in step s-1, finished at the last barrier);
//                           wait copy s+1 (vmcnt leaves the younger ones in flight); BARRIER
//   MFMA wavefronts: BARRIER; for s: multiply stage s % NSTAGE; wait until the stage's LDS reads have returned; BARRIER
//
// Division of the work.  The products of a call (dX, dW or both) form one sequence of units, a unit being one
// 64-wide contraction step of one tile: problem after problem, tile after tile (the tiles of one row of tiles
// next to each other), step after step.  The G workgroups of the launch (at most one per CU) cut the sequence
// into G equal runs, so that every CU does the same number of steps whatever the tile counts and contraction
// lengths are; workgroup b takes run v(b) = (b%8)*(G/8) + b/8, which gives each XCD (workgroups are dealt to
// the 8 XCDs in turn) a contiguous eighth of the sequence and so one L2 the operand panels of its tiles.
// A run covers a tile in part at most at its two ends:
//   * the leading steps of a tile (the run ends inside it), or steps from its middle (the whole run lies inside
//     one tile): the wavefront's partial sums go to the workgroup's slot in the workspace, followed by a flag
//     per wavefront.  A run has at most one such piece, so one slot per run suffices;
//   * the trailing steps of a tile: this workgroup owns the tile.  It does that piece last, then every MFMA
//     wavefront waits for the flags of the same wavefront of the runs v' < v that hold the tile's earlier steps,
//     adds their partial sums to its own in ascending order of v' (a fixed order: results do not change from run
//     to run) and writes the tile out.
// A workgroup thus waits only for runs below its own, which finish their pieces when it finishes its own; the
// flags are cleared by the staging launch that precedes every GEMM launch.  The wait is bounded: if a flag has
// not been raised after some seconds the tile is written as NaN, so that every wavefront ends.
// The clamp's derivative (mask of a problem, src != null): element (r, n) of the result is set to zero where
// |src[r, n]| exceeds its range: lim[r / rows_per_lim] for dW (weights: one range per group of rows), lim_all for dX.
struct ClampMask {
    const float *src;
    const float *lim;
    float lim_all;
    int rows_per_lim;
};

struct SkProblem {
    const uint16_t *A, *B;
    int M, Nc, lda, ldb;
    int nsteps;    // contraction length / 64
    int out;       // 0: bf16 C, 1: fp32 C * scale
    float scale;
    void *C;
    int tiles_n;   // tiles along Nc
    ClampMask mask;
};
constexpr int kSkMaxProblems = 2;
constexpr int kSkMaxRuns = 256;       // one run per workgroup, at most one workgroup per CU
constexpr int kSkFlagsPerRun = 8;     // one flag per MFMA wavefront (six used)
struct SkGroup {
    int n;
    long long ustart[kSkMaxProblems + 1];  // first unit of problem i; [n] = length of the sequence
    SkProblem p[kSkMaxProblems];
    float *slots;                          // kSkMaxRuns slots of one tile of floats
    int *flags;                            // kSkMaxRuns * kSkFlagsPerRun, zero before the launch
};

// a piece of a run: steps [s0, s1) of one tile
struct SkPiece {
    int pi, tile, s0, s1, nsteps;
    long long tile_first_unit;
};

__device__ __forceinline__ SkPiece sk_piece_at(const SkGroup &g, long long u, long long hi)
{
    SkPiece q;
    q.pi = (g.n > 1 && u >= g.ustart[1]) ? 1 : 0;
    const long long r = u - g.ustart[q.pi];
    q.nsteps = g.p[q.pi].nsteps;
    q.tile = (int)(r / q.nsteps);
    q.s0 = (int)(r - (long long)q.tile * q.nsteps);
    const long long room = hi - u;
    q.s1 = (q.nsteps - q.s0 <= room) ? q.nsteps : q.s0 + (int)room;
    q.tile_first_unit = u - q.s0;
    return q;
}

// Partial sums and flags travel between workgroups on different XCDs, whose L2 caches are not coherent with each
// other for ordinary accesses.  They are therefore written and read with device-scope accesses (sc1: stores write
// through, loads do not hit a stale line), which needs no write-back or invalidation of a whole L2 (a release or
// acquire fence at device scope does that, and cost 40 us per launch here).  A wavefront's stores have completed
// when its memory counter is back at zero; only then is its flag raised.
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
// the value of the lane whose number differs in bit 0 / bit 1 (inside a quad of lanes; full-rate DPP moves)
__device__ __forceinline__ uint32_t quad_xor1(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true); }
__device__ __forceinline__ uint32_t quad_xor2(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true); }
__device__ __forceinline__ void sk_store4(float4 *p, const v4f &v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ v4f sk_load4(const float4 *p)  // the value may be used after sk_loads_done only
{
    v4f v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
    return v;
}
// waits until *f is raised (device scope); false if it was not within the bound
__device__ __forceinline__ bool sk_wait_flag(const int *f)
{
    for (int it = 0; it < (1 << 22); ++it) {
        if (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return true;
        __builtin_amdgcn_s_sleep(16);
    }
    return false;
}

template <int NSTAGE, bool MASK, int TM, int TN>
__global__ __launch_bounds__(512) void gemm_bf16_sk_kernel(const SkGroup g)
{
    // an MFMA wavefront owns TM x TN blocks of 32 x 32: tiles of 64*TM x 96*TN (128 x 96, or 256 x 192: half the
    // operand bytes per multiply-add out of L2 and LDS)
    constexpr int WN = 3, NPROD = 2;
    constexpr int BM = 64 * TM, BN = 96 * TN, BKB = 128;  // 64 bf16 per step
    constexpr int A_TOTAL = BM / 8, B_TOTAL = BN / 8;
    constexpr int A_PER = A_TOTAL / NPROD, B_PER = B_TOTAL / NPROD, PERP = A_PER + B_PER;
    constexpr int D = NSTAGE - 1;
    constexpr int A_BYTES = BM * BKB, STAGE_BYTES = (BM + BN) * BKB;
    constexpr int SLOT_FLOATS = BM * BN;
    constexpr int NB = TM * TN;  // blocks per wavefront
    static_assert((D - 1) * PERP < 64, "vmcnt has six bits");
    static_assert(TN <= 2 && (NB == 2 || NB % 4 == 0) && NB <= 8, "partial sums are read four blocks at a time; mask bits of a wavefront's blocks: 16 per block in two 64-bit words");
    __shared__ __align__(1024) uint8_t lds[NSTAGE * STAGE_BYTES];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = (int)gridDim.x;
    const int v = (G & 7) ? (int)blockIdx.x : (int)(blockIdx.x & 7) * (G >> 3) + (int)(blockIdx.x >> 3);
    const long long U = g.ustart[g.n];
    const long long lo = U * v / G, hi = U * (v + 1) / G;
    if (lo >= hi) return;  // (the host gives every run at least one unit)

    // The pieces of this run in the order they are done: the run's first piece last if it is the end of a tile
    // whose beginning belongs to other runs.  Both roles walk the same list.
    const SkPiece first = sk_piece_at(g, lo, hi);
    const bool first_last = first.s0 > 0 && first.s1 == first.nsteps;
    const long long u_begin = first_last ? lo + (first.s1 - first.s0) : lo;

    if ((wave & 3) == 3) {
        // ================================ copies ================================
        const int p = wave >> 2;
        auto copy_piece = [&](const SkPiece &q) {
            const SkProblem &P = g.p[q.pi];
            const int tile_m = q.tile / P.tiles_n, tile_n = q.tile - tile_m * P.tiles_n;
            const int M = P.M, Nc = P.Nc, lda = P.lda, ldb = P.ldb;
            const int nsteps = q.s1 - q.s0;
            // addresses: a wavefront-uniform base per piece and step, a 32-bit byte offset per lane and copy
            // (rows of a tile lie less than 2^32 bytes apart: at most 256 rows of at most 2^25 bytes)
            const uint8_t *a_base = reinterpret_cast<const uint8_t *>(P.A + (size_t)tile_m * BM * lda + q.s0 * 64);
            const uint8_t *b_base = reinterpret_cast<const uint8_t *>(P.B + (size_t)tile_n * BN * ldb + q.s0 * 64);
            const int a_last = M - 1 - tile_m * BM, b_last = Nc - 1 - tile_n * BN;
            uint32_t a_off[A_PER], b_off[B_PER];
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                const int blk = i * NPROD + p;
                int row = blk * 8 + (lane >> 3);
                const int kx = (row >> 1) & 7;
                row = row < a_last ? row : a_last;  // rows past the end re-read the last one; outputs masked
                a_off[i] = (uint32_t)row * (uint32_t)(lda * 2) + (((lane & 7) ^ kx) * 16);
            }
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int blk = i * NPROD + p;
                int row = blk * 8 + (lane >> 3);
                const int kx = (row >> 1) & 7;
                // TN == 2: LDS row 64*wn + 32*tn + l holds row 64*wn + 2*l + tn of the tile, so that a lane's two blocks
                // are neighbouring columns of the result (whole 128-byte lines in the write-out, see there)
                if constexpr (TN == 2) row = (row & ~63) + 2 * (row & 31) + ((row >> 5) & 1);
                row = row < b_last ? row : b_last;
                b_off[i] = (uint32_t)row * (uint32_t)(ldb * 2) + (((lane & 7) ^ kx) * 16);
            }
            auto fetch = [&](int step, int stage) {
                const uint32_t st_ = lds_base + stage * STAGE_BYTES;
                const uint8_t *as = a_base + (size_t)step * BKB, *bs = b_base + (size_t)step * BKB;
#pragma unroll
                for (int i = 0; i < A_PER; ++i) copy16_to_lds(as + a_off[i], st_ + (i * NPROD + p) * 1024);
#pragma unroll
                for (int i = 0; i < B_PER; ++i) copy16_to_lds(bs + b_off[i], st_ + A_BYTES + (i * NPROD + p) * 1024);
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
        };
        for (long long u = u_begin; u < hi;) {
            const SkPiece q = sk_piece_at(g, u, hi);
            copy_piece(q);
            u += q.s1 - q.s0;
        }
        if (first_last) copy_piece(first);
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
        b_frag[sub] = A_BYTES + (wn * TN * 32 + l32) * BKB + (((sub * 2 + hf) ^ key) << 4);
    }
    // this wavefront's part of a slot: float4 number ((cidx*NB + block)*4 + q)*64 + lane holds acc[block][4q..4q+3]
    const size_t slot_part = (size_t)cidx * NB * 4 * 64 + lane;

    auto mma_piece = [&](const SkPiece &q) {
        const SkProblem &P = g.p[q.pi];
        const int tile_m = q.tile / P.tiles_n, tile_n = q.tile - tile_m * P.tiles_n;
        const int M = P.M, Nc = P.Nc;
        const int nsteps = q.s1 - q.s0;
        const bool writes_tile = q.s1 == q.nsteps;  // uniform over the workgroup
        v16f acc[TM][TN];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0.0f;
        // The clamp mask of this wavefront's blocks, as one bit per result, formed before the K-loop so that the
        // write-out depends on no load (a load left between the stores makes every store before it be waited for).
        // Per 32 x 32 block four float4 loads: one instruction covers 8 rows x 32 columns, lane l the row l/8 and
        // the four columns 4*(l%8)... of it.  That is not the accumulator's lane layout: every lane turns its 4 x 4
        // values into predicate bits (nibble q = load q), and the lane that holds the result of row 4*hf + 8*q + j,
        // column l32 finds them in lane (4*hf + j)*8 + l32/4, bit 4*q + l32%4.  Rows and columns past the end
        // re-read valid elements; their results are not stored.
        uint64_t outside[2] = {0, 0};  // bit 16*(block%4) + i of word block/4: result i of the block is zeroed
        bool masked = false;
        if constexpr (MASK) {
            masked = writes_tile && P.mask.src != nullptr;
            if (masked && TN == 2) {
                // a lane's two blocks are the columns cc, cc + 1 of its rows: loaded in the accumulator's own layout
                int cc = tile_n * BN + wn * 64 + 2 * l32;
                cc = cc + 1 < Nc ? cc : Nc - 2;
                const bool pair_ok = (Nc & 1) == 0 && (reinterpret_cast<uintptr_t>(P.mask.src) & 7) == 0;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        int r = tile_m * BM + (wm * TM + tm) * 32 + 4 * hf + 8 * (i >> 2) + (i & 3);
                        r = r < M ? r : M - 1;
                        const float *src = P.mask.src + (size_t)r * Nc + cc;
                        float2 mv;
                        if (pair_ok) mv = *reinterpret_cast<const float2 *>(src);
                        else mv = make_float2(src[0], src[1]);
                        const float lim = P.mask.lim ? P.mask.lim[r / P.mask.rows_per_lim] : P.mask.lim_all;
                        const int b0 = tm * TN;
                        outside[b0 >> 2] |= (uint64_t)(fabsf(mv.x) > lim ? 1u : 0u) << ((b0 & 3) * 16 + i);
                        outside[(b0 + 1) >> 2] |= (uint64_t)(fabsf(mv.y) > lim ? 1u : 0u) << (((b0 + 1) & 3) * 16 + i);
                    }
            } else if (masked) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        int cc = tile_n * BN + (wn * TN + tn) * 32 + 4 * (lane & 7);
                        cc = cc < Nc ? cc : Nc - 4;
                        uint32_t wbits = 0;
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd) {
                            int r = tile_m * BM + (wm * TM + tm) * 32 + 8 * qd + (lane >> 3);
                            r = r < M ? r : M - 1;
                            const float4 mv = *reinterpret_cast<const float4 *>(P.mask.src + (size_t)r * Nc + cc);
                            const float lim = P.mask.lim ? P.mask.lim[r / P.mask.rows_per_lim] : P.mask.lim_all;
                            wbits |= (fabsf(mv.x) > lim ? 1u : 0u) << (4 * qd);
                            wbits |= (fabsf(mv.y) > lim ? 2u : 0u) << (4 * qd);
                            wbits |= (fabsf(mv.z) > lim ? 4u : 0u) << (4 * qd);
                            wbits |= (fabsf(mv.w) > lim ? 8u : 0u) << (4 * qd);
                        }
                        const int blk = tm * TN + tn;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const uint32_t gb = (uint32_t)__shfl((int)wbits, (4 * hf + j) * 8 + (l32 >> 2)) >> (l32 & 3);
#pragma unroll
                            for (int qd = 0; qd < 4; ++qd)
                                outside[blk >> 2] |= (uint64_t)((gb >> (4 * qd)) & 1u) << ((blk & 3) * 16 + 4 * qd + j);
                        }
                    }
            }
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        int stage = 0;
        for (int s = 0; s < nsteps; ++s) {
            const uint8_t *st_ = lds + stage * STAGE_BYTES;
            if constexpr (NB <= 2) {
                // every fragment read of the step first (their latency paid once), then the MFMAs
                v8bf af[4][TM], bf[4][TN];
#pragma unroll
                for (int sub = 0; sub < 4; ++sub) {
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) bf[sub][tn] = *reinterpret_cast<const v8bf *>(st_ + b_frag[sub] + tn * 32 * BKB);
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) af[sub][tm] = *reinterpret_cast<const v8bf *>(st_ + a_frag[sub] + tm * 32 * BKB);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int sub = 0; sub < 4; ++sub)
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn)
                            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[sub][tm], bf[sub][tn], acc[tm][tn], 0, 0, 0);
            } else {
                // a quarter of the step (16 of the 64 features) at a time: the next quarter's fragments are read while
                // the MFMAs of this one run
                v8bf af[2][TM], bf[2][TN];
                auto read_quarter = [&](int sub, int set) {
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) bf[set][tn] = *reinterpret_cast<const v8bf *>(st_ + b_frag[sub] + tn * 32 * BKB);
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) af[set][tm] = *reinterpret_cast<const v8bf *>(st_ + a_frag[sub] + tm * 32 * BKB);
                };
                read_quarter(0, 0);
#pragma unroll
                for (int sub = 0; sub < 4; ++sub) {
                    if (sub < 3) read_quarter(sub + 1, (sub + 1) & 1);
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn)
                            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[sub & 1][tm], bf[sub & 1][tn], acc[tm][tn], 0, 0, 0);
                }
            }
            stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
            // The stage just read is overwritten by copies that the copy wavefronts start right behind the barrier, so
            // this wavefront's reads of it must have returned, not only been issued: the compiler lets the MFMAs that
            // consume the step's last fragments follow below the barrier, and without the explicit wait a wavefront
            // arrives with those reads still queued in the LDS.  (Found as wrong results when another stream's kernel
            // kept the CU's LDS busy; the wait costs 1-2 % per layer.)
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        if (!writes_tile) {
            // partial sums of the tile's leading or middle steps: to this run's slot, then the wavefront's flag
            float4 *slot = reinterpret_cast<float4 *>(g.slots + (size_t)v * SLOT_FLOATS) + slot_part;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        const v4f t = {acc[tm][tn][4 * qd], acc[tm][tn][4 * qd + 1], acc[tm][tn][4 * qd + 2], acc[tm][tn][4 * qd + 3]};
                        sk_store4(slot + ((tm * TN + tn) * 4 + qd) * 64, t);
                    }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // every lane's stores have completed
            if (lane == 0)
                __hip_atomic_store(g.flags + v * kSkFlagsPerRun + cidx, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        if (q.s0 > 0) {
            // the tile's earlier steps were done by the runs below this one: the first of them is the run that holds
            // the tile's first unit
            int w = (int)(q.tile_first_unit * G / U);
            while (U * (w + 1) / G <= q.tile_first_unit) ++w;
            bool ok = true;
            for (; w < v; ++w) {
                ok = sk_wait_flag(g.flags + w * kSkFlagsPerRun + cidx) && ok;
                asm volatile("" ::: "memory");
                const float4 *slot = reinterpret_cast<const float4 *>(g.slots + (size_t)w * SLOT_FLOATS) + slot_part;
                // up to four blocks' worth of loads in flight (their latency is what this costs), then one wait; its
                // operands tie every later use of the values to it
                constexpr int CB = NB < 4 ? NB : 4;
#pragma unroll
                for (int b0 = 0; b0 < NB; b0 += CB) {
                    v4f t[CB][4];
#pragma unroll
                    for (int b = 0; b < CB; ++b)
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd) t[b][qd] = sk_load4(slot + ((b0 + b) * 4 + qd) * 64);
                    if constexpr (CB == 2)
                        asm volatile("s_waitcnt vmcnt(0)"
                                     : "+v"(t[0][0]), "+v"(t[0][1]), "+v"(t[0][2]), "+v"(t[0][3]), "+v"(t[1][0]), "+v"(t[1][1]),
                                       "+v"(t[1][2]), "+v"(t[1][3])::"memory");
                    else
                        asm volatile("s_waitcnt vmcnt(0)"
                                     : "+v"(t[0][0]), "+v"(t[0][1]), "+v"(t[0][2]), "+v"(t[0][3]), "+v"(t[1][0]), "+v"(t[1][1]),
                                       "+v"(t[1][2]), "+v"(t[1][3]), "+v"(t[2][0]), "+v"(t[2][1]), "+v"(t[2][2]), "+v"(t[2][3]),
                                       "+v"(t[3][0]), "+v"(t[3][1]), "+v"(t[3][2]), "+v"(t[3][3])::"memory");
#pragma unroll
                    for (int b = 0; b < CB; ++b) {
                        const int tm = (b0 + b) / TN, tn = (b0 + b) % TN;
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd) {
                            acc[tm][tn][4 * qd] += t[b][qd][0];
                            acc[tm][tn][4 * qd + 1] += t[b][qd][1];
                            acc[tm][tn][4 * qd + 2] += t[b][qd][2];
                            acc[tm][tn][4 * qd + 3] += t[b][qd][3];
                        }
                    }
                }
            }
            if (!ok) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[tm][tn][i] = __builtin_nanf("");
            }
        }
        if constexpr (MASK) {
            // applied as selects before the store loop: inside the bounds-checked store loop the compiler turns the
            // same test into a branch per element (seventy instructions per store instead of eleven)
            if (masked) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const int blk = tm * TN + tn;
                            acc[tm][tn][i] = ((outside[blk >> 2] >> ((blk & 3) * 16 + i)) & 1ull) ? 0.0f : acc[tm][tn][i];
                        }
            }
        }
        const bool interior = (tile_m + 1) * BM <= M && (tile_n + 1) * BN <= Nc;  // uniform over the workgroup
        const float scale = P.scale;
        void *__restrict__ Cout = P.C;
        const bool as_bf16 = P.out == 0;
        const int lq = lane & 3, odd = lane & 1, hi2 = (lane >> 1) & 1;
        if constexpr (TN == 2) {
            // A lane's two blocks are the columns n, n + 1 of its rows (the copies placed the operand rows so).
            const int n = tile_n * BN + wn * 64 + 2 * l32;
            const bool wide_ok = (Nc & 7) == 0 && (reinterpret_cast<uintptr_t>(Cout) & 15) == 0;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int r0 = tile_m * BM + (wm * TM + tm) * 32 + 4 * hf;
                if (interior && wide_ok && as_bf16) {
                    // bf16: the two columns make one 32-bit word per row; four neighbouring lanes then exchange words
                    // (two butterfly steps inside the quad) so that each holds one row of eight columns and writes
                    // 16 bytes: a store instruction covers whole 128-byte lines, and there are 4 of them per 32 rows
                    // instead of 32 two-byte ones.
                    uint16_t *row0 = static_cast<uint16_t *>(Cout) + (size_t)(r0 + lq) * Nc + (n - 2 * lq);
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        uint32_t d[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            d[j] = (uint32_t)f32_to_bf16_rne(acc[tm][0][4 * qd + j]) | ((uint32_t)f32_to_bf16_rne(acc[tm][1][4 * qd + j]) << 16);
                        const uint32_t rx0 = quad_xor1(odd ? d[0] : d[1]), rx1 = quad_xor1(odd ? d[2] : d[3]);
                        const uint32_t e_lo = odd ? rx0 : d[0], e_hi = odd ? d[1] : rx0;  // row odd: this lane pair's words
                        const uint32_t f_lo = odd ? rx1 : d[2], f_hi = odd ? d[3] : rx1;  // row 2 + odd
                        const uint32_t s_lo = quad_xor2(hi2 ? e_lo : f_lo), s_hi = quad_xor2(hi2 ? e_hi : f_hi);
                        v4u o;
                        o[0] = hi2 ? s_lo : e_lo;
                        o[1] = hi2 ? s_hi : e_hi;
                        o[2] = hi2 ? f_lo : s_lo;
                        o[3] = hi2 ? f_hi : s_hi;
                        __builtin_nontemporal_store(o, reinterpret_cast<v4u *>(row0 + (size_t)(8 * qd) * Nc));
                    }
                } else if (interior && wide_ok) {
                    // fp32: 8 bytes per lane and row, 256 contiguous bytes per row and instruction
                    float *blk0 = static_cast<float *>(Cout) + (size_t)r0 * Nc + n;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        v2f o;
                        o[0] = acc[tm][0][i] * scale;
                        o[1] = acc[tm][1][i] * scale;
                        __builtin_nontemporal_store(o, reinterpret_cast<v2f *>(blk0 + (size_t)(8 * (i >> 2) + (i & 3)) * Nc));
                    }
                } else {
#pragma unroll
                    for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const int r = r0 + 8 * (i >> 2) + (i & 3);
                            if (r < M && n + tn < Nc) {
                                const size_t at = (size_t)r * Nc + n + tn;
                                if (as_bf16) static_cast<uint16_t *>(Cout)[at] = f32_to_bf16_rne(acc[tm][tn][i]);
                                else static_cast<float *>(Cout)[at] = acc[tm][tn][i] * scale;
                            }
                        }
                }
            }
        } else {
        const bool packed_ok = (Nc & 3) == 0 && (reinterpret_cast<uintptr_t>(Cout) & 7) == 0;  // 8-byte stores of whole quads
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int r0 = tile_m * BM + (wm * TM + tm) * 32 + 4 * hf;
                const int n = tile_n * BN + (wn * TN + tn) * 32 + l32;
                if (interior) {  // no per-element checks, one base address per block
                    const size_t at0 = (size_t)r0 * Nc + n;
                    // results that no kernel of this call reads again are streamed past the caches
                    if (as_bf16 && packed_ok) {
                        // A lane holds four consecutive rows of one column; four neighbouring lanes exchange values
                        // (two butterfly steps inside the quad) so that each holds one row of four columns and writes
                        // 8 bytes: a quarter of the store instructions.
                        uint16_t *row0 = static_cast<uint16_t *>(Cout) + at0 + (size_t)lq * Nc - lq;
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd) {
                            const uint32_t h0 = f32_to_bf16_rne(acc[tm][tn][4 * qd]), h1 = f32_to_bf16_rne(acc[tm][tn][4 * qd + 1]);
                            const uint32_t h2 = f32_to_bf16_rne(acc[tm][tn][4 * qd + 2]), h3 = f32_to_bf16_rne(acc[tm][tn][4 * qd + 3]);
                            const uint32_t r0x = quad_xor1(odd ? h0 : h1), r1x = quad_xor1(odd ? h2 : h3);
                            const uint32_t w0 = odd ? (r0x | (h1 << 16)) : (h0 | (r0x << 16));  // row odd, this lane pair's columns
                            const uint32_t w1 = odd ? (r1x | (h3 << 16)) : (h2 | (r1x << 16));  // row 2 + odd
                            const uint32_t rx = quad_xor2(hi2 ? w0 : w1);
                            v2u o;
                            o[0] = hi2 ? rx : w0;
                            o[1] = hi2 ? w1 : rx;
                            __builtin_nontemporal_store(o, reinterpret_cast<v2u *>(row0 + (size_t)(8 * qd) * Nc));
                        }
                    } else if (as_bf16) {
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            __builtin_nontemporal_store(f32_to_bf16_rne(acc[tm][tn][i]),
                                                        static_cast<uint16_t *>(Cout) + at0 + (size_t)(8 * (i >> 2) + (i & 3)) * Nc);
                    } else {
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            __builtin_nontemporal_store(acc[tm][tn][i] * scale,
                                                        static_cast<float *>(Cout) + at0 + (size_t)(8 * (i >> 2) + (i & 3)) * Nc);
                    }
                    continue;
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int r = r0 + 8 * (i >> 2) + (i & 3);
                    if (r < M && n < Nc) {
                        const size_t at = (size_t)r * Nc + n;
                        if (as_bf16) static_cast<uint16_t *>(Cout)[at] = f32_to_bf16_rne(acc[tm][tn][i]);
                        else static_cast<float *>(Cout)[at] = acc[tm][tn][i] * scale;
                    }
                }
            }
        }
    };
    for (long long u = u_begin; u < hi;) {
        const SkPiece q = sk_piece_at(g, u, hi);
        mma_piece(q);
        u += q.s1 - q.s0;
    }
    if (first_last) mma_piece(first);
}

// appends a product to a call's list: tiles of 64*TM x 96*TN, the contraction Kc a multiple of 64
template <int TM, int TN>
void sk_add(SkGroup &g, const uint16_t *A, const uint16_t *B, int M, int Nc, int Kc, int lda, int ldb, int out, float scale,
            void *C, const ClampMask *mask)
{
    if (g.n == 0) g.ustart[0] = 0;
    SkProblem &P = g.p[g.n];
    P.A = A; P.B = B; P.M = M; P.Nc = Nc; P.lda = lda; P.ldb = ldb; P.nsteps = Kc / 64; P.out = out; P.scale = scale; P.C = C;
    P.tiles_n = (Nc + 96 * TN - 1) / (96 * TN);
    P.mask = mask ? *mask : ClampMask{nullptr, nullptr, 0.0f, 1};
    const long long tiles = (long long)((M + 64 * TM - 1) / (64 * TM)) * P.tiles_n;
    g.ustart[g.n + 1] = g.ustart[g.n] + tiles * P.nsteps;
    ++g.n;
}

// One launch for the list: one workgroup per CU, every workgroup at least kSkMinUnits steps.
constexpr int kSkMinUnits = 4;
template <int NSTAGE, int TM, int TN>
void sk_launch(const SkGroup &g, hipStream_t st)
{
    const long long U = g.ustart[g.n];
    long long grid = U / kSkMinUnits;
    if (grid > kSkMaxRuns) grid = kSkMaxRuns;
    if (grid < 1) grid = 1;
    if (grid >= 8) grid &= ~7ll;
    bool any_mask = false;
    for (int i = 0; i < g.n; ++i) any_mask = any_mask || g.p[i].mask.src != nullptr;
    if (any_mask)
        hipLaunchKernelGGL((gemm_bf16_sk_kernel<NSTAGE, true, TM, TN>), dim3((unsigned)grid), dim3(512), 0, st, g);
    else
        hipLaunchKernelGGL((gemm_bf16_sk_kernel<NSTAGE, false, TM, TN>), dim3((unsigned)grid), dim3(512), 0, st, g);
}

// One product of a call, as the host sees it
struct SkProduct {
    const uint16_t *A, *B;
    int M, Nc, Kc, lda, ldb, out;
    float scale;
    void *C;
    const ClampMask *mask;
};
// Tiles of 128 x 192 when that leaves every CU at least kSkWideMinSteps of their steps, else 128 x 96; three stages.
constexpr int kSkWideMinSteps = 16;
constexpr size_t kSkSlotBytes = (size_t)128 * 192 * 4;
void sk_run(const SkProduct *prod, int n, float *slots, int *flags, hipStream_t st)
{
    long long wide_units = 0;
    for (int i = 0; i < n; ++i)
        wide_units += (long long)((prod[i].M + 127) / 128) * ((prod[i].Nc + 191) / 192) * (prod[i].Kc / 64);
    SkGroup g;
    g.n = 0;
    g.slots = slots;
    g.flags = flags;
    if (wide_units >= (long long)kSkMaxRuns * kSkWideMinSteps) {
        for (int i = 0; i < n; ++i)
            sk_add<2, 2>(g, prod[i].A, prod[i].B, prod[i].M, prod[i].Nc, prod[i].Kc, prod[i].lda, prod[i].ldb, prod[i].out,
                         prod[i].scale, prod[i].C, prod[i].mask);
        sk_launch<3, 2, 2>(g, st);
    } else {
        for (int i = 0; i < n; ++i)
            sk_add<2, 1>(g, prod[i].A, prod[i].B, prod[i].M, prod[i].Nc, prod[i].Kc, prod[i].lda, prod[i].ldb, prod[i].out,
                         prod[i].scale, prod[i].C, prod[i].mask);
        sk_launch<3, 2, 1>(g, st);
    }
}

struct BwdPlan {
    int64_t Np, Tp;
    size_t off_wt, off_dyp, off_dyt, off_xt, off_slots, off_flags, total;
};

BwdPlan make_plan(int64_t T, int64_t N, int64_t K)
{
    BwdPlan p;
    p.Np = round_up(N, 64);
    p.Tp = round_up(T, 64);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
    p.off_wt = take((size_t)K * p.Np * 2);
    p.off_dyp = take(N % 64 ? (size_t)T * p.Np * 2 : 0);
    p.off_dyt = take((size_t)N * p.Tp * 2);
    p.off_xt = take((size_t)K * p.Tp * 2);
    p.off_slots = take((size_t)kSkMaxRuns * kSkSlotBytes);  // partial sums of tiles shared between workgroups
    p.off_flags = take((size_t)kSkMaxRuns * kSkFlagsPerRun * 4);
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
        a.flags = reinterpret_cast<int *>(ws + p.off_flags); a.n_flags = kSkMaxRuns * kSkFlagsPerRun;
        const dim3 grid((unsigned)(a.nb_w + a.nb_y + a.nb_x + 1));
        switch (bits) {
            case 2: hipLaunchKernelGGL(stage_operands_kernel<2>, grid, dim3(256), 0, st, a); break;
            case 3: hipLaunchKernelGGL(stage_operands_kernel<3>, grid, dim3(256), 0, st, a); break;
            case 4: hipLaunchKernelGGL(stage_operands_kernel<4>, grid, dim3(256), 0, st, a); break;
            default: hipLaunchKernelGGL(stage_operands_kernel<8>, grid, dim3(256), 0, st, a); break;
        }
    }
    // both products in one launch, the workgroups sharing their steps evenly
    SkProduct prod[2];
    int np = 0;
    const ClampMask mx{X, nullptr, clip, 1}, mw{W, m, 0.0f, rpg};
    if (dX) {
        const uint16_t *Aop = dY;
        if (N % 64) {
            uint16_t *dYp = reinterpret_cast<uint16_t *>(ws + p.off_dyp);
            hipLaunchKernelGGL(pad_rows_kernel, dim3((unsigned)((T * Np + 255) / 256)), dim3(256), 0, st, dY, T, (int)N, Np, dYp);
            Aop = dYp;
        }
        prod[np++] = SkProduct{Aop, WT, (int)T, (int)K, Np, Np, Np, 0, 1.0f, dX, X ? &mx : nullptr};
    }
    if (dW) prod[np++] = SkProduct{dYT, XT, (int)N, (int)K, Tp, Tp, Tp, 1, clip / 255.0f, dW, W ? &mw : nullptr};
    sk_run(prod, np, reinterpret_cast<float *>(ws + p.off_slots), reinterpret_cast<int *>(ws + p.off_flags), st);
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
