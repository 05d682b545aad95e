// Quantize / pack kernels for gfx950: group-wise k-bit weights, 8-bit activations (static clip or a
// max-abs range per token), the unpack test hook and the 4/8-bit column-grouped embedding table.
//
// All of them are bound by HBM traffic.  The weight kernel therefore reads each fp32 weight
// from memory exactly once: a team of threads (a workgroup, or a half or a quarter of one) owns
// one group (a contiguous block of N/G rows), keeps it in registers between the max-abs reduction
// and the quantization, and routes the codes through LDS only to regroup them into the 32-code
// slots of the packed layout; resident workgroups walk over the groups of up to 48 matrices.
//
// Every floating-point step that decides a code is a single correctly rounded binary32
// operation (add, divide, round-half-even), in the order the paper's appendix gives them
// (X' - q0, / Delta, round), so the codes do not depend on how the work is split over lanes.
#include "qb_common.hpp"
#include <type_traits>

namespace qb {
namespace {

__device__ __forceinline__ float absmax4(const float4 v, float mx)
{
    return fmaxf(fmaxf(fmaxf(mx, fabsf(v.x)), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w)));
}

// floor(e / d) for 0 <= e < 2^22 without an integer divide; inv = 1/d rounded.
__device__ __forceinline__ int fast_div(int e, int d, float inv)
{
    int q = (int)((float)e * inv);
    if ((q + 1) * d <= e) ++q;
    if (q * d > e) --q;
    return q;
}

// Barrier between the phases of a panel.  BARE: for the streaming kernel, whose copies of the next group into LDS
// (issued as inline assembly, unknown to the compiler) must stay in flight across the phases: only this wavefront's
// LDS operations are awaited (lgkmcnt 0), then a bare s_barrier; __syncthreads() would also wait for the copies.
template <bool BARE>
__device__ __forceinline__ void panel_sync()
{
    if constexpr (BARE) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else __syncthreads();
}

// A team of `threads` threads (a whole workgroup, or a 64-multiple part of one: `tid` is the thread's number in
// the team and `smem` the team's own LDS) quantizes and packs a panel of `prow` consecutive rows that lie inside
// one group, from the panel's weights in registers: float4 number tid + i*threads of the panel in v[i]; mx (and mn
// if ASYM) the thread's share of the range.  Every team of a workgroup must come here (the barriers are the
// workgroup's).  FUSED: the panel is the whole group, the range is found here and m/h are written.  Otherwise m was
// found before and only the panel starting a group writes h.
// LDS: prow rows of (K + 16) code bytes, then prow int32 row sums, then 2*threads/64 floats.
// ASYM: the group's range is [q0, q0 + L*Delta] with q0 in m[g] and Delta in h[g]: read (found before) if !FUSED,
// found here as the group's minimum and fl(fl(max - min)/L) and written if FUSED.
// PARK: the thread's float4 numbers V .. V+PARK-1 wait in LDS (park[p * park_stride]) instead of registers.
template <int BITS, int V, bool FUSED, bool ASYM, bool BARE, int PARK = 0>
__device__ __forceinline__ void panel_finish(
    float4 (&v)[V], float mx, float mn, const int tid, const int threads, int K, int rows_per_group, int prow, float inv_K,
    float inv_prow, uint8_t *__restrict__ packed, float *__restrict__ h, float *__restrict__ m,
    int32_t *__restrict__ rs_w, int panel, uint8_t *smem, const float *__restrict__ clamp_hi,
    const float4 *park = nullptr, int park_stride = 0)
{
    static_assert(PARK == 0 || (FUSED && !ASYM), "parked weights: the symmetric one-pass form only");
    // clamp_hi (ASYM, !FUSED): the range was given by the caller as [m[g], clamp_hi[g]]; weights outside are clamped
    const int stride = K + 16;
    int *rowsum = reinterpret_cast<int *>(smem + (size_t)prow * stride);
    float *red = reinterpret_cast<float *>(rowsum + prow);
    const int row0 = panel * prow;  // first row of the panel
    const int g = row0 / rows_per_group;
    const int n4 = prow * (K >> 2);
    constexpr float Lf = (float)((1 << BITS) - 1);

    for (int r = tid; r < prow; r += threads) rowsum[r] = 0;

    float mg, dg = 0.0f;
    if (FUSED) {
        const int nw = threads >> 6;
        mx = wave_max(mx);
        if constexpr (ASYM) mn = -wave_max(-mn);
        if ((tid & 63) == 0) {
            red[tid >> 6] = mx;
            if constexpr (ASYM) red[nw + (tid >> 6)] = mn;
        }
        panel_sync<BARE>();
        mg = red[0];
        for (int w = 1; w < nw; ++w) mg = fmaxf(mg, red[w]);
        if constexpr (ASYM) {
            float lo = red[nw];
            for (int w = 1; w < nw; ++w) lo = fminf(lo, red[nw + w]);
            dg = __fdiv_rn(__fsub_rn(mg, lo), Lf);
            mg = lo;
        }
    } else {
        mg = m[g];
        if constexpr (ASYM) dg = h[g];
        panel_sync<BARE>();
    }
    Quantizer qz;
    if constexpr (ASYM) qz.set_range(mg, dg);
    else qz.set(mg, Lf);
    if (tid == 0 && row0 % rows_per_group == 0) {
        if constexpr (ASYM) {
            if (FUSED) {
                h[g] = dg;
                m[g] = mg;
            }
        } else {
            h[g] = qz.half_step();
            if (FUSED) m[g] = mg;
        }
    }
    if constexpr (!FUSED && ASYM) {
        if (clamp_hi) {  // a given range [lo, hi]: X' = Clamp(X, lo, hi)
            const float hi = clamp_hi[g];
#pragma unroll
            for (int i = 0; i < V; ++i) {
                v[i].x = __builtin_amdgcn_fmed3f(v[i].x, mg, hi);
                v[i].y = __builtin_amdgcn_fmed3f(v[i].y, mg, hi);
                v[i].z = __builtin_amdgcn_fmed3f(v[i].z, mg, hi);
                v[i].w = __builtin_amdgcn_fmed3f(v[i].w, mg, hi);
            }
        }
    }
    if (!FUSED && !ASYM) {  // the range was given: it may be smaller than the group's max-abs (clipped range)
#pragma unroll
        for (int i = 0; i < V; ++i) {
            v[i].x = __builtin_amdgcn_fmed3f(v[i].x, -mg, mg);
            v[i].y = __builtin_amdgcn_fmed3f(v[i].y, -mg, mg);
            v[i].z = __builtin_amdgcn_fmed3f(v[i].z, -mg, mg);
            v[i].w = __builtin_amdgcn_fmed3f(v[i].w, -mg, mg);
        }
    }

    // codes, four per dword, into the LDS image of the panel.  Row and column of a thread's float4 advance by a fixed
    // step from one to the next (no division per float4), and the test `fast` is taken once for the group.
    {
        const int step = 4 * threads;
        const int dr = fast_div(step, K, inv_K), dc = step - dr * K;  // uniform
        int r = fast_div(tid << 2, K, inv_K);
        int c = (tid << 2) - r * K;
        auto walk = [&](auto fast_tag) {
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const int idx = tid + i * threads;
                if (idx < n4)
                    *reinterpret_cast<uint32_t *>(smem + (size_t)(r * stride + c)) = qz.template code4t<decltype(fast_tag)::value>(v[i]);
                r += dr;
                c += dc;
                if (c >= K) {
                    c -= K;
                    ++r;
                }
            }
#pragma unroll
            for (int p = 0; p < PARK; ++p) {
                const int idx = tid + (V + p) * threads;
                if (idx < n4)
                    *reinterpret_cast<uint32_t *>(smem + (size_t)(r * stride + c)) =
                        qz.template code4t<decltype(fast_tag)::value>(park[p * park_stride]);
                r += dr;
                c += dc;
                if (c >= K) {
                    c -= K;
                    ++r;
                }
            }
        };
        if (qz.fast) walk(std::true_type{});
        else walk(std::false_type{});
    }
    panel_sync<BARE>();

    // regroup into 32-code slots; consecutive threads take consecutive rows of one column run
    const int nruns = prow * (K >> 5);
    for (int id = tid; id < nruns; id += threads) {
        const int rc = fast_div(id, prow, inv_prow);
        const int r = id - rc * prow;
        const uint4 lo = *reinterpret_cast<const uint4 *>(smem + (size_t)r * stride + rc * 32);
        const uint4 hi = *reinterpret_cast<const uint4 *>(smem + (size_t)r * stride + rc * 32 + 16);
        const uint32_t d[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        uint32_t sum = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) sum = __builtin_amdgcn_sad_u8(d[i], 0u, sum);
        atomicAdd(&rowsum[r], (int)sum);
        uint32_t out[BITS];
        pack_run<BITS>(d, out);
        uint32_t *dst = reinterpret_cast<uint32_t *>(packed + slot_index(row0 + r, rc, K) * (size_t)(4 * BITS));
        if constexpr (BITS == 8) {
            reinterpret_cast<uint4 *>(dst)[0] = make_uint4(out[0], out[1], out[2], out[3]);
            reinterpret_cast<uint4 *>(dst)[1] = make_uint4(out[4], out[5], out[6], out[7]);
        } else if constexpr (BITS == 4) {
            reinterpret_cast<uint4 *>(dst)[0] = make_uint4(out[0], out[1], out[2], out[3]);
        } else if constexpr (BITS == 2) {
            reinterpret_cast<uint2 *>(dst)[0] = make_uint2(out[0], out[1]);
        } else {
            dst[0] = out[0];
            dst[1] = out[1];
            dst[2] = out[2];
        }
    }
    panel_sync<BARE>();
    for (int r = tid; r < prow; r += threads) rs_w[row0 + r] = rowsum[r] - K * (1 << (BITS - 1));
}

// One workgroup, one panel: the panel's weights are read from global memory into registers, then panel_finish.
template <int BITS, int THREADS, int V, bool FUSED, bool ASYM = false>
__device__ __forceinline__ void quantize_panel_body(
    const float *__restrict__ W, int K, int rows_per_group, int prow, float inv_K, float inv_prow,
    uint8_t *__restrict__ packed, float *__restrict__ h, float *__restrict__ m, int32_t *__restrict__ rs_w,
    int panel, uint8_t *smem, const float *__restrict__ clamp_hi = nullptr)
{
    const int tid = threadIdx.x;
    const int row0 = panel * prow;
    const float4 *src = reinterpret_cast<const float4 *>(W + (size_t)row0 * K);
    const int n4 = prow * (K >> 2);
    float4 v[V];
    float mx = 0.0f, mn = 0.0f;
    if constexpr (FUSED && ASYM) mx = mn = W[(size_t)row0 * K];  // any element of the group
#pragma unroll
    for (int i = 0; i < V; ++i) {
        const int idx = tid + i * THREADS;
        if (idx < n4) {
            v[i] = src[idx];
            if constexpr (FUSED && ASYM) {
                mx = fmaxf(fmaxf(mx, fmaxf(v[i].x, v[i].y)), fmaxf(v[i].z, v[i].w));
                mn = fminf(fminf(mn, fminf(v[i].x, v[i].y)), fminf(v[i].z, v[i].w));
            } else if (FUSED) {
                mx = absmax4(v[i], mx);
            }
        }
    }
    panel_finish<BITS, V, FUSED, ASYM, false>(v, mx, mn, tid, THREADS, K, rows_per_group, prow, inv_K, inv_prow, packed, h, m,
                                              rs_w, panel, smem, clamp_hi);
}

template <int BITS, int THREADS, int V, bool FUSED, bool ASYM = false>
__global__ __launch_bounds__(THREADS) void quantize_panel_kernel(
    const float *__restrict__ W, int K, int rows_per_group, int prow, float inv_K, float inv_prow,
    uint8_t *__restrict__ packed, float *__restrict__ h, float *__restrict__ m, int32_t *__restrict__ rs_w,
    const float *__restrict__ clamp_hi)
{
    extern __shared__ __align__(16) uint8_t smem[];
    quantize_panel_body<BITS, THREADS, V, FUSED, ASYM>(W, K, rows_per_group, prow, inv_K, inv_prow, packed, h, m, rs_w,
                                                       blockIdx.x, smem, clamp_hi);
}

// ---- asymmetric ranges: min and max of every group.  Floats are mapped to unsigned keys that order like the
// floats (sign bit flipped for non-negative values, all bits flipped for negative ones), so that slices of a
// group combine through integer atomic max / min.  hi_key must start at 0, lo_key at 0xffffffff.
__device__ __forceinline__ uint32_t float_key(float f)
{
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}
__global__ void range_init_kernel(uint32_t *hi_key, uint32_t *lo_key, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        hi_key[i] = 0u;
        lo_key[i] = 0xffffffffu;
    }
}
__global__ __launch_bounds__(256) void minmax_slices_kernel(const float *__restrict__ W, int64_t group_elems, int slices,
                                                            uint32_t *__restrict__ hi_key, uint32_t *__restrict__ lo_key)
{
    __shared__ float red[8];
    const int g = blockIdx.x / slices, s = blockIdx.x % slices;
    const int64_t n4 = group_elems >> 2;
    const int64_t per = (n4 + slices - 1) / slices;
    const int64_t lo = (int64_t)s * per, hi = (lo + per < n4) ? lo + per : n4;
    const float4 *src = reinterpret_cast<const float4 *>(W + (int64_t)g * group_elems);
    if (lo >= hi) return;  // (uniform per workgroup)
    float mx = src[lo].x, mn = mx;
    for (int64_t i = lo + threadIdx.x; i < hi; i += 256) {
        const float4 v = src[i];
        mx = fmaxf(fmaxf(mx, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
        mn = fminf(fminf(mn, fminf(v.x, v.y)), fminf(v.z, v.w));
    }
    mx = wave_max(mx);
    mn = -wave_max(-mn);
    if ((threadIdx.x & 63) == 0) {
        red[threadIdx.x >> 6] = mx;
        red[4 + (threadIdx.x >> 6)] = mn;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        mn = fminf(fminf(red[4], red[5]), fminf(red[6], red[7]));
        atomicMax(hi_key + g, float_key(mx));
        atomicMin(lo_key + g, float_key(mn));
    }
}
// keys -> q0 = min and Delta = fl(fl(max - min)/L), in place
__global__ void range_finish_kernel(float *delta, float *q0, int n, float L)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const float hi = key_float(reinterpret_cast<const uint32_t *>(delta)[i]);
        const float lo = key_float(reinterpret_cast<const uint32_t *>(q0)[i]);
        delta[i] = __fdiv_rn(__fsub_rn(hi, lo), L);
        q0[i] = lo;
    }
}

// given ranges [lo, hi] -> q0 = lo and Delta = fl(fl(hi - lo)/L)
__global__ void range_given_kernel(const float *__restrict__ lo, const float *__restrict__ hi, float *delta, float *q0, int n,
                                   float L)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        delta[i] = __fdiv_rn(__fsub_rn(hi[i], lo[i]), L);
        q0[i] = lo[i];
    }
}

constexpr int kMaxFusedElems = 1024 * 4 * 8;  // one group in the registers of 1024 threads, 8 float4 each

// Several matrices in one launch (a fine-tuning step re-quantizes every matrix of the model):
// workgroup w serves group w - first_wg[j] of job j.  Passed by value as the kernel argument.
constexpr int kQuantBatch = 48;  // jobs of one launch: the descriptor below is the kernel argument (under 4 KB)
struct QuantBatch {
    int n;
    int first_wg[kQuantBatch + 1];
    const float *W[kQuantBatch];
    uint8_t *packed[kQuantBatch];
    float *h[kQuantBatch];
    float *m[kQuantBatch];
    int32_t *rs_w[kQuantBatch];
    int K[kQuantBatch];
    int rows_per_group[kQuantBatch];
    int bits[kQuantBatch];
    float inv_K[kQuantBatch];
    float inv_rows[kQuantBatch];
    int per_item[kQuantBatch];    // groups per work item (first_wg counts items)
    uint32_t team_bytes[kQuantBatch];  // LDS of one team of the job
};

// Resident workgroups walk over work items: item w is `per_item` (1, 2 or 4) consecutive groups of one matrix, one
// group per team of THREADS/per_item threads, so that small groups do not leave most of a workgroup idle.
// Why resident: a workgroup has no loads in flight while it computes, and workgroups that start together share the
// memory bandwidth evenly and so finish loading together: launched one per group they stay in step through their two
// or three rounds and the memory system idles for about a third of the time (measured with timestamps per phase).
// Walking over many items, the workgroups of a CU drift apart and loads of some run under the arithmetic of others.
template <int THREADS, int V, int PARK, int MIN_WAVES>
__global__ __launch_bounds__(THREADS, MIN_WAVES) void quantize_batched_kernel(const QuantBatch b, uint32_t park_off)
{
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr int LOG_THREADS = THREADS == 1024 ? 10 : THREADS == 512 ? 9 : 8;
    static_assert(THREADS == 1 << LOG_THREADS, "256, 512 or 1024 threads");
    const int total = b.first_wg[b.n];
    int j = 0;  // the job of the item: items come in rising order, so the search goes on from the last one
    for (int item = blockIdx.x; item < total; item += gridDim.x) {
        while (j + 1 < b.n && item >= b.first_wg[j + 1]) ++j;
        const int per = b.per_item[j];
        const int sh = LOG_THREADS - (per >> 1), threads = 1 << sh;  // per is 1, 2 or 4: teams of whole wavefronts
        const int team = threadIdx.x >> sh, tid = threadIdx.x & (threads - 1);
        const int rpg = b.rows_per_group[j], K = b.K[j];
        const int n4 = rpg * (K >> 2);                                // float4 of a group
        const int g = (item - b.first_wg[j]) * per + team;
        const float4 *src = reinterpret_cast<const float4 *>(b.W[j]) + (size_t)g * n4;
        float4 v[V];
        float mx = 0.0f;
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const int idx = tid + i * threads;
            if (idx < n4) {
                v[i] = src[idx];
                mx = absmax4(v[i], mx);
            }
        }
        // V float4 stay in registers, PARK more wait in LDS (behind every team's area), so that 64 registers a thread do
        float4 *park = reinterpret_cast<float4 *>(smem + park_off) + threadIdx.x;
#pragma unroll
        for (int p = 0; p < PARK; ++p) {
            const int idx = tid + (V + p) * threads;
            if (idx < n4) {
                const float4 x = src[idx];
                mx = absmax4(x, mx);
                park[p * THREADS] = x;
            }
        }
        uint8_t *lds = smem + (size_t)team * b.team_bytes[j];
        switch (b.bits[j]) {
            case 2: panel_finish<2, V, true, false, false, PARK>(v, mx, 0.0f, tid, threads, K, rpg, rpg, b.inv_K[j], b.inv_rows[j], b.packed[j], b.h[j], b.m[j], b.rs_w[j], g, lds, nullptr, park, THREADS); break;
            case 3: panel_finish<3, V, true, false, false, PARK>(v, mx, 0.0f, tid, threads, K, rpg, rpg, b.inv_K[j], b.inv_rows[j], b.packed[j], b.h[j], b.m[j], b.rs_w[j], g, lds, nullptr, park, THREADS); break;
            case 4: panel_finish<4, V, true, false, false, PARK>(v, mx, 0.0f, tid, threads, K, rpg, rpg, b.inv_K[j], b.inv_rows[j], b.packed[j], b.h[j], b.m[j], b.rs_w[j], g, lds, nullptr, park, THREADS); break;
            default: panel_finish<8, V, true, false, false, PARK>(v, mx, 0.0f, tid, threads, K, rpg, rpg, b.inv_K[j], b.inv_rows[j], b.packed[j], b.h[j], b.m[j], b.rs_w[j], g, lds, nullptr, park, THREADS); break;
        }
        __syncthreads();  // the row sums were read to the end before the next item clears them
    }
}

// Two-pass path for groups too large for one workgroup's registers: slices of a group reduce
// |w| and combine through an integer atomic max on the bit pattern (order-preserving for
// non-negative floats).  m must have been zero-filled.
__global__ __launch_bounds__(256) void absmax_slices_kernel(const float *__restrict__ W, int64_t group_elems,
                                                            int slices, float *__restrict__ m)
{
    __shared__ float red[4];
    const int g = blockIdx.x / slices, s = blockIdx.x % slices;
    const int64_t n4 = group_elems >> 2;
    const int64_t per = (n4 + slices - 1) / slices;
    const int64_t lo = (int64_t)s * per, hi = (lo + per < n4) ? lo + per : n4;
    const float4 *src = reinterpret_cast<const float4 *>(W + (int64_t)g * group_elems);
    float mx = 0.0f;
    for (int64_t i = lo + threadIdx.x; i < hi; i += 256) mx = absmax4(src[i], mx);
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        atomicMax(reinterpret_cast<unsigned int *>(m) + g, __float_as_uint(mx));
    }
}

__global__ void fill_zero_kernel(float *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

// ---- activations: a wavefront walks over token rows (row = wavefront id, + number of wavefronts, ...)
// in chunks of 256 float4; the loads of the next chunk (possibly of the next row) are in flight while
// the current one is quantized, so the memory pipe never drains between rows.
template <bool DEVCLIP>
__global__ __launch_bounds__(256) void quantize_act_kernel(const float *__restrict__ X, int T, int K, float clip,
                                                           const float *__restrict__ clip_dev,
                                                           int8_t *__restrict__ Xq, int32_t *__restrict__ rs_x,
                                                           float *__restrict__ hx_rows)
{
    if constexpr (DEVCLIP) clip = *clip_dev;  // the range found by tensor_absmax_kernel
    const int lane = threadIdx.x & 63;
    const int nwaves = gridDim.x * 4;
    int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= T) return;
    Quantizer qz;
    qz.set(clip, 255.0f);
    const int k4 = K >> 2;
    const int chunks = (k4 + 255) >> 8;

    float4 cur[4], nxt[4];
    auto load = [&](float4 (&v)[4], int r, int c) {
        const float4 *src = reinterpret_cast<const float4 *>(X + (size_t)r * K);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = (c << 8) + u * 64 + lane;
            if (idx < k4) v[u] = src[idx];
        }
    };
    load(cur, row, 0);
    uint32_t sum = 0;
    int c = 0;
    while (true) {
        // where the next chunk is
        int nrow = row, nc = c + 1;
        if (nc == chunks) { nc = 0; nrow = row + nwaves; }
        const bool more = nrow < T;
        if (more) load(nxt, nrow, nc);
        uint32_t *dst = reinterpret_cast<uint32_t *>(Xq + (size_t)row * K);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = (c << 8) + u * 64 + lane;
            if (idx < k4) {
                float4 v = cur[u];
                v.x = __builtin_amdgcn_fmed3f(v.x, -clip, clip);
                v.y = __builtin_amdgcn_fmed3f(v.y, -clip, clip);
                v.z = __builtin_amdgcn_fmed3f(v.z, -clip, clip);
                v.w = __builtin_amdgcn_fmed3f(v.w, -clip, clip);
                const uint32_t q = qz.code4(v);
                sum = __builtin_amdgcn_sad_u8(q, 0u, sum);
                dst[idx] = q ^ 0x80808080u;  // u - 128 as int8
            }
        }
        if (nc == 0) {  // row finished
            const int total = wave_sum((int)sum);
            if (lane == 0) {
                rs_x[row] = total - 128 * K;
                if constexpr (DEVCLIP) hx_rows[row] = qz.half_step();
            }
            sum = 0;
        }
        if (!more) break;
        row = nrow;
        c = nc;
#pragma unroll
        for (int u = 0; u < 4; ++u) cur[u] = nxt[u];
    }
}

// Several activation tensors in one launch (the inputs of a layer's linears): the rows of all tensors form one
// sequence that the wavefronts walk through as quantize_act_kernel walks through the rows of one tensor, the next
// chunk (possibly of another tensor) in flight while the current one is quantized.
struct ActBatch {
    int n;
    int row_start[QB_MAX_BATCH + 1];  // first row of tensor i in the sequence; [n] = number of rows
    const float *X[QB_MAX_BATCH];
    int8_t *Xq[QB_MAX_BATCH];
    int32_t *rs_x[QB_MAX_BATCH];
    int K[QB_MAX_BATCH];
    float clip[QB_MAX_BATCH];
};

__global__ __launch_bounds__(256) void quantize_act_batched_kernel(const ActBatch b)
{
    const int lane = threadIdx.x & 63;
    const int nwaves = gridDim.x * 4;
    const int total = b.row_start[b.n];
    int vrow = blockIdx.x * 4 + (threadIdx.x >> 6);  // position in the sequence of rows (uniform over the wavefront)
    if (vrow >= total) return;
    auto job_of = [&](int r) {
        int j = 0;
        while (j + 1 < b.n && r >= b.row_start[j + 1]) ++j;
        return j;
    };
    int j = job_of(vrow);
    int K = b.K[j], k4 = K >> 2, chunks = (k4 + 255) >> 8;
    float clip = b.clip[j];
    Quantizer qz;
    qz.set(clip, 255.0f);

    float4 cur[4], nxt[4];
    auto load = [&](float4 (&v)[4], int jj, int r, int c) {
        const int kk4 = b.K[jj] >> 2;
        const float4 *src = reinterpret_cast<const float4 *>(b.X[jj] + (size_t)(r - b.row_start[jj]) * b.K[jj]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = (c << 8) + u * 64 + lane;
            if (idx < kk4) v[u] = src[idx];
        }
    };
    load(cur, j, vrow, 0);
    uint32_t sum = 0;
    int c = 0;
    while (true) {
        int nrow = vrow, nc = c + 1, nj = j;
        if (nc == chunks) {
            nc = 0;
            nrow = vrow + nwaves;
            if (nrow < total) nj = job_of(nrow);
        }
        const bool more = nrow < total;
        if (more) load(nxt, nj, nrow, nc);
        const int row = vrow - b.row_start[j];
        uint32_t *dst = reinterpret_cast<uint32_t *>(b.Xq[j] + (size_t)row * K);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = (c << 8) + u * 64 + lane;
            if (idx < k4) {
                float4 v = cur[u];
                v.x = __builtin_amdgcn_fmed3f(v.x, -clip, clip);
                v.y = __builtin_amdgcn_fmed3f(v.y, -clip, clip);
                v.z = __builtin_amdgcn_fmed3f(v.z, -clip, clip);
                v.w = __builtin_amdgcn_fmed3f(v.w, -clip, clip);
                const uint32_t q = qz.code4(v);
                sum = __builtin_amdgcn_sad_u8(q, 0u, sum);
                dst[idx] = q ^ 0x80808080u;  // u - 128 as int8
            }
        }
        if (nc == 0) {  // row finished
            const int tot = wave_sum((int)sum);
            if (lane == 0) b.rs_x[j][row] = tot - 128 * K;
            sum = 0;
        }
        if (!more) break;
        if (nj != j) {  // the next row belongs to another tensor
            j = nj;
            K = b.K[j];
            k4 = K >> 2;
            chunks = (k4 + 255) >> 8;
            clip = b.clip[j];
            qz.set(clip, 255.0f);
        }
        vrow = nrow;
        c = nc;
#pragma unroll
        for (int u = 0; u < 4; ++u) cur[u] = nxt[u];
    }
}

// ---- activations with one range for the whole tensor, c = max |X|: pass 1 reduces into a device float
// (zero-filled before; non-negative floats order like their bit patterns, so an integer atomic max serves),
// pass 2 is quantize_act_kernel reading its clip from that float.
__global__ __launch_bounds__(1024) void tensor_absmax_kernel(const float4 *__restrict__ X, int64_t n4,
                                                             float *__restrict__ c)
{
    // few, large workgroups: the atomics of all workgroups meet at one address, which takes them one at a time
    __shared__ float part[16];
    const int64_t stride = (int64_t)gridDim.x * 1024;
    int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    float mx = 0.0f;
    for (; i + 3 * stride < n4; i += 4 * stride) {  // four loads in flight
        const float4 a = X[i], b = X[i + stride], d = X[i + 2 * stride], e = X[i + 3 * stride];
        mx = absmax4(a, mx);
        mx = absmax4(b, mx);
        mx = absmax4(d, mx);
        mx = absmax4(e, mx);
    }
    for (; i < n4; i += stride) mx = absmax4(X[i], mx);
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x < 64) {
        mx = wave_max(threadIdx.x < 16 ? part[threadIdx.x] : 0.0f);
        if (threadIdx.x == 0) atomicMax(reinterpret_cast<unsigned int *>(c), __float_as_uint(mx));
    }
}

// ---- activations with a range per token: c_t = max_j |X[t,j]|.  One wavefront per row; the row's first
// 64*V float4 stay in registers between the max and the quantization, the rest (K > 256*V) is read again.
template <int V>
__global__ __launch_bounds__(256) void quantize_act_dyn_kernel(const float *__restrict__ X, int T, int K,
                                                               int8_t *__restrict__ Xq, int32_t *__restrict__ rs_x,
                                                               float *__restrict__ hx)
{
    const int lane = threadIdx.x & 63;
    const int nwaves = gridDim.x * 4;
    const int k4 = K >> 2;
    for (int row = blockIdx.x * 4 + (threadIdx.x >> 6); row < T; row += nwaves) {
        const float4 *src = reinterpret_cast<const float4 *>(X + (size_t)row * K);
        float4 v[V];
        float mx = 0.0f;
#pragma unroll
        for (int u = 0; u < V; ++u) {
            const int idx = u * 64 + lane;
            if (idx < k4) {
                v[u] = src[idx];
                mx = absmax4(v[u], mx);
            }
        }
        for (int idx = V * 64 + lane; idx < k4; idx += 64) mx = absmax4(src[idx], mx);
        const float c = wave_max(mx);
        Quantizer qz;
        qz.set(c, 255.0f);
        if (lane == 0) hx[row] = qz.half_step();
        uint32_t *dst = reinterpret_cast<uint32_t *>(Xq + (size_t)row * K);
        uint32_t sum = 0;
#pragma unroll
        for (int u = 0; u < V; ++u) {
            const int idx = u * 64 + lane;
            if (idx < k4) {
                const uint32_t q = qz.code4(v[u]);
                sum = __builtin_amdgcn_sad_u8(q, 0u, sum);
                dst[idx] = q ^ 0x80808080u;  // u - 128 as int8
            }
        }
        for (int idx = V * 64 + lane; idx < k4; idx += 64) {
            const uint32_t q = qz.code4(src[idx]);
            sum = __builtin_amdgcn_sad_u8(q, 0u, sum);
            dst[idx] = q ^ 0x80808080u;
        }
        const int total = wave_sum((int)sum);
        if (lane == 0) rs_x[row] = total - 128 * K;
    }
}

// ---- test hook: slots -> row-major codes -----------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(256) void unpack_codes_kernel(const uint8_t *__restrict__ packed, int N, int K,
                                                           uint8_t *__restrict__ codes)
{
    const int runs = K >> 5;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= (int64_t)N * runs) return;
    const int n = (int)(id / runs), rc = (int)(id % runs);
    const uint32_t *src = reinterpret_cast<const uint32_t *>(packed + slot_index(n, rc, K) * (size_t)(4 * BITS));
    uint32_t in[BITS], d[8];
#pragma unroll
    for (int i = 0; i < BITS; ++i) in[i] = src[i];
    unpack_run<BITS>(in, d);
    uint4 *dst = reinterpret_cast<uint4 *>(codes + (size_t)n * K + rc * 32);
    dst[0] = make_uint4(d[0], d[1], d[2], d[3]);
    dst[1] = make_uint4(d[4], d[5], d[6], d[7]);
}

// ---- embedding table: groups are column blocks --------------------------------------------------------
// pass 1: a workgroup takes EMB_ROWS rows of up to 1024 columns; each thread owns four columns, keeps eight
// row loads in flight, and the workgroup combines per group in LDS before it touches m (zero-filled before;
// max-abs values are non-negative floats, which order like their bit patterns).
constexpr int EMB_ROWS = 32;
__global__ __launch_bounds__(256) void embedding_absmax_kernel(const float *__restrict__ E, int64_t V, int d,
                                                               int cols_per_group, float *__restrict__ m)
{
    __shared__ unsigned int gm[1024];
    const int d4 = d >> 2;
    const int c4 = blockIdx.x * 256 + threadIdx.x;
    const int col_lo = blockIdx.x * 1024;
    const int col_hi = (col_lo + 1024 < d) ? col_lo + 1024 : d;  // exclusive
    const int g_lo = col_lo / cols_per_group, g_n = (col_hi - 1) / cols_per_group - g_lo + 1;
    for (int i = threadIdx.x; i < g_n; i += 256) gm[i] = 0u;
    __syncthreads();
    if (c4 < d4) {
        const int64_t r0 = (int64_t)blockIdx.y * EMB_ROWS;
        const int nr = (int)((V - r0 < EMB_ROWS) ? V - r0 : EMB_ROWS);
        const float4 *src = reinterpret_cast<const float4 *>(E) + r0 * d4 + c4;
        float4 mx = make_float4(0.f, 0.f, 0.f, 0.f);
        auto take = [&](const float4 v) {
            mx.x = fmaxf(mx.x, fabsf(v.x));
            mx.y = fmaxf(mx.y, fabsf(v.y));
            mx.z = fmaxf(mx.z, fabsf(v.z));
            mx.w = fmaxf(mx.w, fabsf(v.w));
        };
        int r = 0;
        for (; r + 8 <= nr; r += 8) {
            float4 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = src[(int64_t)(r + i) * d4];
#pragma unroll
            for (int i = 0; i < 8; ++i) take(v[i]);
        }
        for (; r < nr; ++r) take(src[(int64_t)r * d4]);
        const int c = c4 << 2;
        const int g0 = c / cols_per_group - g_lo, g3 = (c + 3) / cols_per_group - g_lo;
        if (g0 == g3) {
            atomicMax(gm + g0, __float_as_uint(fmaxf(fmaxf(mx.x, mx.y), fmaxf(mx.z, mx.w))));
        } else {
            atomicMax(gm + g0, __float_as_uint(mx.x));
            atomicMax(gm + (c + 1) / cols_per_group - g_lo, __float_as_uint(mx.y));
            atomicMax(gm + (c + 2) / cols_per_group - g_lo, __float_as_uint(mx.z));
            atomicMax(gm + g3, __float_as_uint(mx.w));
        }
    }
    __syncthreads();
    unsigned int *mb = reinterpret_cast<unsigned int *>(m);
    for (int i = threadIdx.x; i < g_n; i += 256)
        if (gm[i] != 0u) atomicMax(mb + g_lo + i, gm[i]);
}

// pass 2: codes, and h = m/L.  Same tiling; a thread sets up the quantizers of its four columns once.
// BITS = 8: one code per byte.  BITS = 4: two per byte, column 2i in the low nibble of byte i (a row is the
// little-endian bit stream of its codes).
template <int BITS>
__global__ __launch_bounds__(256) void embedding_quantize_kernel(const float *__restrict__ E, int64_t V, int d,
                                                                 int cols_per_group, int groups,
                                                                 const float *__restrict__ m, float *__restrict__ h,
                                                                 uint8_t *__restrict__ codes)
{
    constexpr float Lf = (float)((1 << BITS) - 1);
    if (blockIdx.x == 0 && blockIdx.y == 0) {
        for (int g = threadIdx.x; g < groups; g += 256) {
            const float mg = m[g];
            h[g] = (mg == 0.0f) ? 0.0f : __fdiv_rn(mg, Lf);
        }
    }
    const int d4 = d >> 2;
    const int c4 = blockIdx.x * 256 + threadIdx.x;
    if (c4 >= d4) return;
    const int c = c4 << 2;
    Quantizer qz[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int g = (c + i) / cols_per_group;
        if (i > 0 && g == (c + i - 1) / cols_per_group) qz[i] = qz[i - 1];
        else qz[i].set(m[g], Lf);
    }
    const int64_t r0 = (int64_t)blockIdx.y * EMB_ROWS;
    const int nr = (int)((V - r0 < EMB_ROWS) ? V - r0 : EMB_ROWS);
    const float4 *src = reinterpret_cast<const float4 *>(E) + r0 * d4 + c4;
    auto code4 = [&](const float4 v) {
        uint32_t q = __builtin_amdgcn_cvt_pk_u8_f32(qz[0].code_f(v.x), 0, 0u);
        q = __builtin_amdgcn_cvt_pk_u8_f32(qz[1].code_f(v.y), 1, q);
        q = __builtin_amdgcn_cvt_pk_u8_f32(qz[2].code_f(v.z), 2, q);
        return __builtin_amdgcn_cvt_pk_u8_f32(qz[3].code_f(v.w), 3, q);
    };
    if constexpr (BITS == 8) {
        uint32_t *dst = reinterpret_cast<uint32_t *>(codes) + r0 * d4 + c4;
        int r = 0;
        for (; r + 8 <= nr; r += 8) {
            float4 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = src[(int64_t)(r + i) * d4];
#pragma unroll
            for (int i = 0; i < 8; ++i) __builtin_nontemporal_store(code4(v[i]), dst + (int64_t)(r + i) * d4);
        }
        for (; r < nr; ++r) dst[(int64_t)r * d4] = code4(src[(int64_t)r * d4]);
    } else {
        // four codes (one per byte of q) -> two bytes: low nibbles from bytes 0 and 2, high from bytes 1 and 3
        auto nib4 = [&](const float4 v) {
            const uint32_t q = code4(v);
            return (uint16_t)((q & 0xFu) | ((q >> 4) & 0xF0u) | ((q >> 8) & 0xF00u) | ((q >> 12) & 0xF000u));
        };
        uint16_t *dst = reinterpret_cast<uint16_t *>(codes) + r0 * d4 + c4;
        int r = 0;
        for (; r + 8 <= nr; r += 8) {
            float4 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = src[(int64_t)(r + i) * d4];
#pragma unroll
            for (int i = 0; i < 8; ++i) dst[(int64_t)(r + i) * d4] = nib4(v[i]);
        }
        for (; r < nr; ++r) dst[(int64_t)r * d4] = nib4(src[(int64_t)r * d4]);
    }
}

template <int BITS>
__global__ __launch_bounds__(256) void embedding_gather_kernel(const uint8_t *__restrict__ codes,
                                                               const float *__restrict__ h, int64_t V, int d,
                                                               int cols_per_group, const int64_t *__restrict__ ids,
                                                               int64_t n_ids, float *__restrict__ out)
{
    constexpr int L = (1 << BITS) - 1;
    const int d4 = d >> 2;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= n_ids * d4) return;
    const int64_t i = id / d4;
    const int c = (int)(id % d4) << 2;
    const int64_t tok = ids[i];
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    if (tok >= 0 && tok < V) {
        int u0, u1, u2, u3;
        if constexpr (BITS == 8) {
            const uint32_t q = *reinterpret_cast<const uint32_t *>(codes + tok * d + c);
            u0 = q & 255u; u1 = (q >> 8) & 255u; u2 = (q >> 16) & 255u; u3 = q >> 24;
        } else {
            const uint32_t q = *reinterpret_cast<const uint16_t *>(codes + ((tok * d + c) >> 1));
            u0 = q & 15u; u1 = (q >> 4) & 15u; u2 = (q >> 8) & 15u; u3 = (q >> 12) & 15u;
        }
        o.x = h[(c + 0) / cols_per_group] * (float)(2 * u0 - L);
        o.y = h[(c + 1) / cols_per_group] * (float)(2 * u1 - L);
        o.z = h[(c + 2) / cols_per_group] * (float)(2 * u2 - L);
        o.w = h[(c + 3) / cols_per_group] * (float)(2 * u3 - L);
    }
    reinterpret_cast<float4 *>(out)[id] = o;
}


template <int BITS, int THREADS, bool ASYM = false>
void launch_panel(const float *W, int K, int rows_per_group, int prow, int panels, uint8_t *packed, float *h, float *m,
                  int32_t *rs_w, hipStream_t st, const float *clamp_hi = nullptr)
{
    const size_t lds = (size_t)prow * (K + 16) + (size_t)prow * 4 + 128;
    hipLaunchKernelGGL((quantize_panel_kernel<BITS, THREADS, 8, false, ASYM>), dim3(panels), dim3(THREADS), lds, st, W, K,
                       rows_per_group, prow, 1.0f / (float)K, 1.0f / (float)prow, packed, h, m, rs_w, clamp_hi);
}

// groups too large for one workgroup's registers: max-abs by slices, then panels of whole rows
template <int BITS>
qb_status quantize_two_pass(const float *W, int64_t N, int64_t K, int groups, uint8_t *packed, float *h, float *m,
                            int32_t *rs_w, hipStream_t st)
{
    const int rpg = (int)(N / groups);
    const int64_t gelems = (int64_t)rpg * K;
    int prow = 1;
    for (int p = rpg; p >= 1; --p)
        if (rpg % p == 0 && (int64_t)p * K <= kMaxFusedElems) { prow = p; break; }
    const int slices = (int)((gelems + 65535) / 65536);
    hipLaunchKernelGGL(fill_zero_kernel, dim3((groups + 255) / 256), dim3(256), 0, st, m, groups);
    hipLaunchKernelGGL(absmax_slices_kernel, dim3(groups * slices), dim3(256), 0, st, W, gelems, slices, m);
    const int64_t pelems = (int64_t)prow * K;
    if (pelems <= 8192) launch_panel<BITS, 256>(W, (int)K, rpg, prow, (int)(N / prow), packed, h, m, rs_w, st);
    else if (pelems <= 16384) launch_panel<BITS, 512>(W, (int)K, rpg, prow, (int)(N / prow), packed, h, m, rs_w, st);
    else launch_panel<BITS, 1024>(W, (int)K, rpg, prow, (int)(N / prow), packed, h, m, rs_w, st);
    return launch_status();
}

// ranges given by the caller: the second pass alone
template <int BITS>
qb_status quantize_given_range(const float *W, int64_t N, int64_t K, int groups, const float *m_in, uint8_t *packed,
                               float *h, int32_t *rs_w, hipStream_t st)
{
    const int rpg = (int)(N / groups);
    int prow = 1;
    for (int p = rpg; p >= 1; --p)
        if (rpg % p == 0 && (int64_t)p * K <= kMaxFusedElems) { prow = p; break; }
    float *m = const_cast<float *>(m_in);  // read only on this path
    const int64_t pelems = (int64_t)prow * K;
    if (pelems <= 8192) launch_panel<BITS, 256>(W, (int)K, rpg, prow, (int)(N / prow), packed, h, m, rs_w, st);
    else if (pelems <= 16384) launch_panel<BITS, 512>(W, (int)K, rpg, prow, (int)(N / prow), packed, h, m, rs_w, st);
    else launch_panel<BITS, 1024>(W, (int)K, rpg, prow, (int)(N / prow), packed, h, m, rs_w, st);
    return launch_status();
}

// asymmetric ranges: fused when a group fits one workgroup; else keys, min/max by slices, Delta and q0, then the panels
template <int BITS>
qb_status quantize_asym(const float *W, int64_t N, int64_t K, int groups, uint8_t *packed, float *delta, float *q0,
                        int32_t *rs_w, hipStream_t st)
{
    const int rpg = (int)(N / groups);
    const int64_t gelems = (int64_t)rpg * K;
    if (gelems <= kMaxFusedElems) {  // a group fits one workgroup's registers: one pass, one launch
        const size_t lds = (size_t)rpg * (K + 16) + (size_t)rpg * 4 + 128;
        const float inv_K = 1.0f / (float)K, inv_rows = 1.0f / (float)rpg;
        const dim3 grid(groups);
        if (gelems <= 256 * 4 * 8)
            hipLaunchKernelGGL((quantize_panel_kernel<BITS, 256, 8, true, true>), grid, dim3(256), lds, st, W, (int)K, rpg, rpg,
                               inv_K, inv_rows, packed, delta, q0, rs_w, static_cast<const float *>(nullptr));
        else if (gelems <= 512 * 4 * 10)
            hipLaunchKernelGGL((quantize_panel_kernel<BITS, 512, 10, true, true>), grid, dim3(512), lds, st, W, (int)K, rpg, rpg,
                               inv_K, inv_rows, packed, delta, q0, rs_w, static_cast<const float *>(nullptr));
        else
            hipLaunchKernelGGL((quantize_panel_kernel<BITS, 1024, 8, true, true>), grid, dim3(1024), lds, st, W, (int)K, rpg,
                               rpg, inv_K, inv_rows, packed, delta, q0, rs_w, static_cast<const float *>(nullptr));
        return launch_status();
    }
    int prow = 1;
    for (int p = rpg; p >= 1; --p)
        if (rpg % p == 0 && (int64_t)p * K <= kMaxFusedElems) { prow = p; break; }
    const int slices = (int)((gelems + 65535) / 65536);
    const dim3 gg((groups + 255) / 256);
    hipLaunchKernelGGL(range_init_kernel, gg, dim3(256), 0, st, reinterpret_cast<uint32_t *>(delta),
                       reinterpret_cast<uint32_t *>(q0), groups);
    hipLaunchKernelGGL(minmax_slices_kernel, dim3(groups * slices), dim3(256), 0, st, W, gelems, slices,
                       reinterpret_cast<uint32_t *>(delta), reinterpret_cast<uint32_t *>(q0));
    hipLaunchKernelGGL(range_finish_kernel, gg, dim3(256), 0, st, delta, q0, groups, (float)((1 << BITS) - 1));
    const int64_t pelems = (int64_t)prow * K;
    if (pelems <= 8192) launch_panel<BITS, 256, true>(W, (int)K, rpg, prow, (int)(N / prow), packed, delta, q0, rs_w, st);
    else if (pelems <= 16384) launch_panel<BITS, 512, true>(W, (int)K, rpg, prow, (int)(N / prow), packed, delta, q0, rs_w, st);
    else launch_panel<BITS, 1024, true>(W, (int)K, rpg, prow, (int)(N / prow), packed, delta, q0, rs_w, st);
    return launch_status();
}

// asymmetric ranges given by the caller: Delta and q0 from [lo, hi], then panels that clamp to the range
template <int BITS>
qb_status quantize_asym_given(const float *W, int64_t N, int64_t K, int groups, const float *lo, const float *hi,
                              uint8_t *packed, float *delta, float *q0, int32_t *rs_w, hipStream_t st)
{
    const int rpg = (int)(N / groups);
    int prow = 1;
    for (int p = rpg; p >= 1; --p)
        if (rpg % p == 0 && (int64_t)p * K <= kMaxFusedElems) { prow = p; break; }
    hipLaunchKernelGGL(range_given_kernel, dim3((groups + 255) / 256), dim3(256), 0, st, lo, hi, delta, q0, groups,
                       (float)((1 << BITS) - 1));
    const int64_t pelems = (int64_t)prow * K;
    if (pelems <= 8192) launch_panel<BITS, 256, true>(W, (int)K, rpg, prow, (int)(N / prow), packed, delta, q0, rs_w, st, hi);
    else if (pelems <= 16384) launch_panel<BITS, 512, true>(W, (int)K, rpg, prow, (int)(N / prow), packed, delta, q0, rs_w, st, hi);
    else launch_panel<BITS, 1024, true>(W, (int)K, rpg, prow, (int)(N / prow), packed, delta, q0, rs_w, st, hi);
    return launch_status();
}

}  // namespace
}  // namespace qb

using namespace qb;

extern "C" qb_status qb_quantize_groupwise_batched(const qb_quant_job *jobs, int n_jobs, void *stream);

extern "C" qb_status qb_quantize_groupwise_asym_range(const float *W, int64_t N, int64_t K, int bits, int groups,
                                                      const float *lo, const float *hi, void *packed, float *delta,
                                                      float *q0, int32_t *rs_w, void *stream)
{
    if (!W || !lo || !hi || !packed || !delta || !q0 || !rs_w) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (N <= 0 || N > (1 << 24) || !k_ok(K) || groups <= 0 || N % groups != 0) return QB_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *p = static_cast<uint8_t *>(packed);
    switch (bits) {
        case 2: return quantize_asym_given<2>(W, N, K, groups, lo, hi, p, delta, q0, rs_w, st);
        case 3: return quantize_asym_given<3>(W, N, K, groups, lo, hi, p, delta, q0, rs_w, st);
        case 4: return quantize_asym_given<4>(W, N, K, groups, lo, hi, p, delta, q0, rs_w, st);
        default: return quantize_asym_given<8>(W, N, K, groups, lo, hi, p, delta, q0, rs_w, st);
    }
}

extern "C" qb_status qb_quantize_groupwise_asym(const float *W, int64_t N, int64_t K, int bits, int groups, void *packed,
                                                float *delta, float *q0, int32_t *rs_w, void *stream)
{
    if (!W || !packed || !delta || !q0 || !rs_w) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (N <= 0 || N > (1 << 24) || !k_ok(K) || groups <= 0 || N % groups != 0) return QB_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *p = static_cast<uint8_t *>(packed);
    switch (bits) {
        case 2: return quantize_asym<2>(W, N, K, groups, p, delta, q0, rs_w, st);
        case 3: return quantize_asym<3>(W, N, K, groups, p, delta, q0, rs_w, st);
        case 4: return quantize_asym<4>(W, N, K, groups, p, delta, q0, rs_w, st);
        default: return quantize_asym<8>(W, N, K, groups, p, delta, q0, rs_w, st);
    }
}

extern "C" qb_status qb_quantize_groupwise_clip(const float *W, int64_t N, int64_t K, int bits, int groups, const float *m_in,
                                                void *packed, float *h, int32_t *rs_w, void *stream)
{
    if (!W || !m_in || !packed || !h || !rs_w) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (N <= 0 || N > (1 << 24) || !k_ok(K) || groups <= 0 || N % groups != 0) return QB_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *p = static_cast<uint8_t *>(packed);
    switch (bits) {
        case 2: return quantize_given_range<2>(W, N, K, groups, m_in, p, h, rs_w, st);
        case 3: return quantize_given_range<3>(W, N, K, groups, m_in, p, h, rs_w, st);
        case 4: return quantize_given_range<4>(W, N, K, groups, m_in, p, h, rs_w, st);
        default: return quantize_given_range<8>(W, N, K, groups, m_in, p, h, rs_w, st);
    }
}

extern "C" qb_status qb_quantize_groupwise(const float *W, int64_t N, int64_t K, int bits, int groups, void *packed,
                                           float *h, float *m, int32_t *rs_w, void *stream)
{
    if (!W || !packed || !h || !m || !rs_w) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (N <= 0 || N > (1 << 24) || !k_ok(K) || groups <= 0 || N % groups != 0) return QB_ERR_SHAPE;
    if ((N / groups) * K <= kMaxFusedElems) {
        const qb_quant_job job = {W, N, K, bits, groups, packed, h, m, rs_w};
        return qb_quantize_groupwise_batched(&job, 1, stream);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *p = static_cast<uint8_t *>(packed);
    switch (bits) {
        case 2: return quantize_two_pass<2>(W, N, K, groups, p, h, m, rs_w, st);
        case 3: return quantize_two_pass<3>(W, N, K, groups, p, h, m, rs_w, st);
        case 4: return quantize_two_pass<4>(W, N, K, groups, p, h, m, rs_w, st);
        default: return quantize_two_pass<8>(W, N, K, groups, p, h, m, rs_w, st);
    }
}

static qb_status check_quant_job(const qb_quant_job &j)
{
    if (!j.W || !j.packed || !j.h || !j.m || !j.rs_w) return QB_ERR_NULL;
    if (!bits_ok(j.bits)) return QB_ERR_BITS;
    if (j.N <= 0 || j.N > (1 << 24) || !k_ok(j.K) || j.groups <= 0 || j.N % j.groups != 0) return QB_ERR_SHAPE;
    return QB_OK;
}

// How many consecutive groups of a job one work item takes (one team of threads/per threads each): at most per_cap,
// as many as the teams' registers (cap float4 a thread) and a modest LDS hold.
static int groups_per_item(const qb_quant_job &j, int threads, int cap, int per_cap)
{
    const int rpg = (int)(j.N / j.groups);
    const int64_t gelems = (int64_t)rpg * j.K;
    const size_t team = (size_t)rpg * (j.K + 16) + (size_t)rpg * 4 + 80;
    int per = per_cap;
    while (per > 1 && (j.groups % per != 0 || gelems > (int64_t)(threads / per) * 4 * cap || per * team > 48 * 1024)) per >>= 1;
    return per;
}

extern "C" qb_status qb_quantize_groupwise_batched(const qb_quant_job *jobs, int n_jobs, void *stream)
{
    if (n_jobs < 0) return QB_ERR_SHAPE;
    if (n_jobs == 0) return QB_OK;
    if (!jobs) return QB_ERR_NULL;
    for (int i = 0; i < n_jobs; ++i) {
        const qb_status s = check_quant_job(jobs[i]);
        if (s != QB_OK) return s;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    // A launch has one workgroup size, chosen for its largest group; a group is held in registers.  Measured on
    // BERT-base groups (18432 weights): 512 threads with up to ten float4 each beat 1024 threads with eight (more
    // workgroups per CU in different phases, cheaper barriers).
    int64_t max_elems = 0;
    for (int i = 0; i < n_jobs; ++i) {
        const int64_t gelems = jobs[i].N / jobs[i].groups * jobs[i].K;
        if (gelems <= kMaxFusedElems && gelems > max_elems) max_elems = gelems;
    }
    const int threads = max_elems <= 256 * 4 * 8 ? 256 : max_elems <= 512 * 4 * 10 ? 512 : 1024;
    const int cap = threads == 512 ? 10 : 8;  // float4 per thread
    // groups per work item: 4 if that still leaves every resident workgroup an item, else 2, else 1
    const int resident = 2048 / threads * 256;  // workgroups that fit the 256 CUs at 64 registers a thread
    int per_cap = 4;
    for (; per_cap > 1; per_cap >>= 1) {
        int64_t items = 0;
        for (int i = 0; i < n_jobs; ++i)
            if (jobs[i].N / jobs[i].groups * jobs[i].K <= kMaxFusedElems)
                items += jobs[i].groups / groups_per_item(jobs[i], threads, cap, per_cap);
        if (items >= resident) break;
    }
    QuantBatch b;
    b.n = 0;
    size_t lds = 0;
    auto flush = [&]() {
        if (b.n == 0) return;
        const int items = b.first_wg[b.n];
        const dim3 grid(items < resident ? items : resident);
        const uint32_t park_off = (uint32_t)lds;
        if (threads == 256) hipLaunchKernelGGL((quantize_batched_kernel<256, 8, 0, 8>), grid, dim3(256), lds, st, b, park_off);
        else if (threads == 512) hipLaunchKernelGGL((quantize_batched_kernel<512, 8, 2, 8>), grid, dim3(512), lds + 2 * 512 * 16, st, b, park_off);
        else hipLaunchKernelGGL((quantize_batched_kernel<1024, 8, 0, 8>), grid, dim3(1024), lds, st, b, park_off);
        b.n = 0; lds = 0;
    };
    for (int i = 0; i < n_jobs; ++i) {
        const qb_quant_job &j = jobs[i];
        const int rpg = (int)(j.N / j.groups);
        const int64_t gelems = (int64_t)rpg * j.K;
        if (gelems > kMaxFusedElems) {  // group too large for one workgroup: the two-pass path, on its own
            const qb_status s = qb_quantize_groupwise(j.W, j.N, j.K, j.bits, j.groups, j.packed, j.h, j.m, j.rs_w, stream);
            if (s != QB_OK) return s;
            continue;
        }
        const size_t team = ((size_t)rpg * (j.K + 16) + (size_t)rpg * 4 + 64 + 15) & ~(size_t)15;  // at most 34 KB
        const int per = groups_per_item(j, threads, cap, per_cap);
        if (b.n == 0) b.first_wg[0] = 0;
        const int k = b.n++;
        b.W[k] = j.W; b.packed[k] = static_cast<uint8_t *>(j.packed); b.h[k] = j.h; b.m[k] = j.m; b.rs_w[k] = j.rs_w;
        b.K[k] = (int)j.K; b.rows_per_group[k] = rpg; b.bits[k] = j.bits;
        b.inv_K[k] = 1.0f / (float)j.K; b.inv_rows[k] = 1.0f / (float)rpg;
        b.per_item[k] = per;
        b.team_bytes[k] = (uint32_t)team;
        b.first_wg[k + 1] = b.first_wg[k] + j.groups / per;
        if (per * team > lds) lds = per * team;
        if (b.n == kQuantBatch) flush();
    }
    flush();
    return launch_status();
}

extern "C" qb_status qb_quantize_act(const float *X, int64_t T, int64_t K, float clip, int8_t *Xq, int32_t *rs_x,
                                     void *stream)
{
    if (!X || !Xq || !rs_x) return QB_ERR_NULL;
    if (T <= 0 || T > (1 << 30) || !k_ok(K)) return QB_ERR_SHAPE;
    if (!(clip > 0.0f) || !(clip < 3.0e38f)) return QB_ERR_CLIP;
    // at most 8 workgroups per CU; fewer rows than that: one wavefront per row
    unsigned blocks = (unsigned)((T + 3) / 4);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(quantize_act_kernel<false>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), X, (int)T,
                       (int)K, clip, static_cast<const float *>(nullptr), Xq, rs_x, static_cast<float *>(nullptr));
    return launch_status();
}

extern "C" qb_status qb_quantize_act_batched(const qb_act_job *jobs, int n_jobs, void *stream)
{
    if (n_jobs < 0) return QB_ERR_SHAPE;
    if (n_jobs == 0) return QB_OK;
    if (!jobs) return QB_ERR_NULL;
    int64_t rows = 0;
    for (int i = 0; i < n_jobs; ++i) {
        const qb_act_job &j = jobs[i];
        if (!j.X || !j.Xq || !j.rs_x) return QB_ERR_NULL;
        if (j.T <= 0 || j.T > (1 << 30) || !k_ok(j.K)) return QB_ERR_SHAPE;
        if (!(j.clip > 0.0f) || !(j.clip < 3.0e38f)) return QB_ERR_CLIP;
        rows += j.T;
    }
    if (rows > (1 << 30)) return QB_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (int i0 = 0; i0 < n_jobs; i0 += QB_MAX_BATCH) {
        ActBatch b;
        b.n = n_jobs - i0 < QB_MAX_BATCH ? n_jobs - i0 : QB_MAX_BATCH;
        b.row_start[0] = 0;
        for (int k = 0; k < b.n; ++k) {
            const qb_act_job &j = jobs[i0 + k];
            b.X[k] = j.X; b.Xq[k] = j.Xq; b.rs_x[k] = j.rs_x; b.K[k] = (int)j.K; b.clip[k] = j.clip;
            b.row_start[k + 1] = b.row_start[k] + (int)j.T;
        }
        unsigned blocks = (unsigned)((b.row_start[b.n] + 3) / 4);
        if (blocks > 2048) blocks = 2048;
        hipLaunchKernelGGL(quantize_act_batched_kernel, dim3(blocks), dim3(256), 0, st, b);
    }
    return launch_status();
}

extern "C" qb_status qb_quantize_act_dyn_tensor(const float *X, int64_t T, int64_t K, int8_t *Xq, int32_t *rs_x,
                                                float *hx_rows, float *c_out, void *stream)
{
    if (!X || !Xq || !rs_x || !hx_rows || !c_out) return QB_ERR_NULL;
    if (T <= 0 || T > (1 << 30) || !k_ok(K)) return QB_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t n4 = T * K / 4;
    unsigned rblocks = (unsigned)((n4 + 4095) / 4096);
    if (rblocks > 256) rblocks = 256;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, st, c_out, 1);
    hipLaunchKernelGGL(tensor_absmax_kernel, dim3(rblocks), dim3(1024), 0, st, reinterpret_cast<const float4 *>(X), n4,
                       c_out);
    unsigned blocks = (unsigned)((T + 3) / 4);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(quantize_act_kernel<true>, dim3(blocks), dim3(256), 0, st, X, (int)T, (int)K, 0.0f,
                       static_cast<const float *>(c_out), Xq, rs_x, hx_rows);
    return launch_status();
}

extern "C" qb_status qb_quantize_act_dyn(const float *X, int64_t T, int64_t K, int8_t *Xq, int32_t *rs_x, float *hx_rows,
                                         void *stream)
{
    if (!X || !Xq || !rs_x || !hx_rows) return QB_ERR_NULL;
    if (T <= 0 || T > (1 << 30) || !k_ok(K)) return QB_ERR_SHAPE;
    unsigned blocks = (unsigned)((T + 3) / 4);
    if (blocks > 2048) blocks = 2048;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (K <= 1024) hipLaunchKernelGGL(quantize_act_dyn_kernel<4>, dim3(blocks), dim3(256), 0, st, X, (int)T, (int)K, Xq, rs_x, hx_rows);
    else hipLaunchKernelGGL(quantize_act_dyn_kernel<16>, dim3(blocks), dim3(256), 0, st, X, (int)T, (int)K, Xq, rs_x, hx_rows);
    return launch_status();
}

extern "C" qb_status qb_unpack_codes(const void *packed, int64_t N, int64_t K, int bits, uint8_t *codes, void *stream)
{
    if (!packed || !codes) return QB_ERR_NULL;
    if (!bits_ok(bits)) return QB_ERR_BITS;
    if (N <= 0 || N > (1 << 24) || !k_ok(K)) return QB_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t *p = static_cast<const uint8_t *>(packed);
    const unsigned blocks = (unsigned)((N * (K / 32) + 255) / 256);
    switch (bits) {
        case 2: hipLaunchKernelGGL(unpack_codes_kernel<2>, dim3(blocks), dim3(256), 0, st, p, (int)N, (int)K, codes); break;
        case 3: hipLaunchKernelGGL(unpack_codes_kernel<3>, dim3(blocks), dim3(256), 0, st, p, (int)N, (int)K, codes); break;
        case 4: hipLaunchKernelGGL(unpack_codes_kernel<4>, dim3(blocks), dim3(256), 0, st, p, (int)N, (int)K, codes); break;
        default: hipLaunchKernelGGL(unpack_codes_kernel<8>, dim3(blocks), dim3(256), 0, st, p, (int)N, (int)K, codes); break;
    }
    return launch_status();
}

extern "C" qb_status qb_embedding_quantize_bits(const float *E, int64_t V, int64_t d, int bits, int groups, uint8_t *codes,
                                                float *h, float *m, void *stream)
{
    if (!E || !codes || !h || !m) return QB_ERR_NULL;
    if (bits != 4 && bits != 8) return QB_ERR_BITS;
    if (V <= 0 || V > (1 << 30) || !k_ok(d) || groups <= 0 || d % groups != 0) return QB_ERR_SHAPE;
    // one workgroup row per EMB_ROWS table rows: the grid's second dimension holds at most 65535 of them
    if ((V + EMB_ROWS - 1) / EMB_ROWS > 65535) return QB_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int cpg = (int)(d / groups);
    const dim3 grid((unsigned)((d / 4 + 255) / 256), (unsigned)((V + EMB_ROWS - 1) / EMB_ROWS));
    hipLaunchKernelGGL(fill_zero_kernel, dim3((groups + 255) / 256), dim3(256), 0, st, m, groups);
    hipLaunchKernelGGL(embedding_absmax_kernel, grid, dim3(256), 0, st, E, V, (int)d, cpg, m);
    if (bits == 8)
        hipLaunchKernelGGL(embedding_quantize_kernel<8>, grid, dim3(256), 0, st, E, V, (int)d, cpg, groups, m, h, codes);
    else
        hipLaunchKernelGGL(embedding_quantize_kernel<4>, grid, dim3(256), 0, st, E, V, (int)d, cpg, groups, m, h, codes);
    return launch_status();
}

extern "C" qb_status qb_embedding_quantize(const float *E, int64_t V, int64_t d, int groups, uint8_t *codes, float *h,
                                           float *m, void *stream)
{
    return qb_embedding_quantize_bits(E, V, d, 8, groups, codes, h, m, stream);
}

extern "C" qb_status qb_embedding_gather_bits(const uint8_t *codes, const float *h, int64_t V, int64_t d, int bits,
                                              int groups, const int64_t *ids, int64_t n_ids, float *out, void *stream)
{
    if (!codes || !h || (n_ids > 0 && (!ids || !out))) return QB_ERR_NULL;
    if (bits != 4 && bits != 8) return QB_ERR_BITS;
    if (V <= 0 || !k_ok(d) || groups <= 0 || d % groups != 0 || n_ids < 0 || n_ids > (1 << 30)) return QB_ERR_SHAPE;
    if (n_ids == 0) return QB_OK;
    const int64_t n4 = n_ids * (d / 4);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bits == 8)
        hipLaunchKernelGGL(embedding_gather_kernel<8>, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, codes, h, V,
                           (int)d, (int)(d / groups), ids, n_ids, out);
    else
        hipLaunchKernelGGL(embedding_gather_kernel<4>, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, codes, h, V,
                           (int)d, (int)(d / groups), ids, n_ids, out);
    return launch_status();
}

extern "C" qb_status qb_embedding_gather(const uint8_t *codes, const float *h, int64_t V, int64_t d, int groups,
                                         const int64_t *ids, int64_t n_ids, float *out, void *stream)
{
    return qb_embedding_gather_bits(codes, h, V, d, 8, groups, ids, n_ids, out, stream);
}
