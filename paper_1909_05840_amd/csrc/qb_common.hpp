// Shared device/host helpers of the gfx950 kernels: wavefront reductions, the private packed
// weight layout, argument checks.  Nothing here is used by the CPU checker under oracle/.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/qbert.h"

namespace qb {

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kRun = 32;           // codes per packed slot (one lane's share of a 64-code unit)
constexpr int kUnit = 64;          // codes per K-unit (= QB_K_ALIGN)
constexpr int kNBlock = QB_N_BLOCK;

// ---- packed weight layout ("slots") ---------------------------------------------------------
// Rows are padded to blocks of 32 output neurons.  For row block cb = n/32 and K-unit ku = j/64
// there are 64 slots, one per lane of a wavefront: lane = 32*hf + n%32 with hf = (j%64)/32.
// Slot (cb, ku, lane) holds the 32 codes u[n][64*ku + 32*hf + 0..31] in 4*bits bytes and sits at
// byte offset ((cb*(K/64) + ku)*64 + lane) * 4*bits, so that one wavefront fetches a whole
// 32-neuron x 64-feature block with one fully coalesced load and every lane ends up holding
// exactly the bytes the int8 MFMA wants from it (no trip through LDS for the weights).
// Inside a slot the codes are bit-sliced so that byte-parallel shifts and masks expand four
// codes at a time:
//   8 bit: byte i = code i
//   4 bit: dword q (0..3), byte j: low nibble = code 8q+j, high nibble = code 8q+4+j
//   2 bit: dword q (0..1), byte j, 2-bit field i (0..3) = code 16q+4i+j
//   3 bit: dwords 0,1 = the low two bits of every code in the 2-bit arrangement,
//          dword 2, byte j, bit i (0..7) = bit 2 of code 4i+j
__host__ __device__ inline int64_t padded_rows(int64_t N) { return (N + kNBlock - 1) / kNBlock * kNBlock; }

__device__ __forceinline__ size_t slot_index(int n, int run, int K)
{
    const int cb = n >> 5, ln = n & 31, ku = run >> 1, hf = run & 1;
    return ((size_t)cb * (size_t)(K >> 6) + (size_t)ku) * 64 + (size_t)(hf * 32 + ln);
}

// d[0..7]: 32 codes, four per dword (code 4i+j in byte j of d[i]) -> out[0..BITS-1]
template <int BITS>
__device__ __forceinline__ void pack_run(const uint32_t (&d)[8], uint32_t (&out)[BITS])
{
    if constexpr (BITS == 8) {
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = d[i];
    } else if constexpr (BITS == 4) {
#pragma unroll
        for (int q = 0; q < 4; ++q) out[q] = d[2 * q] | (d[2 * q + 1] << 4);
    } else if constexpr (BITS == 2) {
#pragma unroll
        for (int q = 0; q < 2; ++q)
            out[q] = d[4 * q] | (d[4 * q + 1] << 2) | (d[4 * q + 2] << 4) | (d[4 * q + 3] << 6);
    } else {
        static_assert(BITS == 3, "bits");
        uint32_t hi = 0;
#pragma unroll
        for (int q = 0; q < 2; ++q)
            out[q] = (d[4 * q] & 0x03030303u) | ((d[4 * q + 1] & 0x03030303u) << 2) |
                     ((d[4 * q + 2] & 0x03030303u) << 4) | ((d[4 * q + 3] & 0x03030303u) << 6);
#pragma unroll
        for (int i = 0; i < 8; ++i) hi |= ((d[i] >> 2) & 0x01010101u) << i;
        out[2] = hi;
    }
}

// inverse of pack_run: in[0..BITS-1] -> d[0..7] (codes 0..L, four per dword)
template <int BITS>
__device__ __forceinline__ void unpack_run(const uint32_t (&in)[BITS], uint32_t (&d)[8])
{
    if constexpr (BITS == 8) {
#pragma unroll
        for (int i = 0; i < 8; ++i) d[i] = in[i];
    } else if constexpr (BITS == 4) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            d[2 * q] = in[q] & 0x0F0F0F0Fu;
            d[2 * q + 1] = (in[q] >> 4) & 0x0F0F0F0Fu;
        }
    } else if constexpr (BITS == 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i) d[i] = (in[i >> 2] >> (2 * (i & 3))) & 0x03030303u;
    } else {
        static_assert(BITS == 3, "bits");
#pragma unroll
        for (int i = 0; i < 8; ++i)
            d[i] = ((in[i >> 2] >> (2 * (i & 3))) & 0x03030303u) | (((in[2] >> i) & 0x01010101u) << 2);
    }
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// The quantizer of one range [-m, +m] (q0 = -m): code = clamp(rint(fl((w + m) / Delta)), 0, L),
// every step one correctly rounded binary32 operation.
//
// The division is the expensive step (these kernels have ~20 ALU operations per element to spend
// at HBM speed), so the common case multiplies by rinv = fl(1/Delta) instead, and falls back to
// the true division exactly when the two could disagree:
//   t  = fl(s/Delta)  = (s/Delta)(1+e3),           |e| <= 2^-24 each
//   t' = fl(s*rinv)   = (s/Delta)(1+e1)(1+e2)
//   |t' - t| <= (s/Delta) * 3.0001 * 2^-24 <= 255.0001 * 3.0001 * 2^-24 < 4.6e-5
// (s/Delta <= L(1+2^-23) <= 255.0001).  With n = rint(t') and d = t' - n (exact by Sterbenz),
// |d| <= 0.4999 puts t' at least 1e-4 away from every half-integer, hence t strictly on the same
// side of it: rint(t) = n, and no tie is involved.  Otherwise the lane redoes the step with the
// IEEE division.  `fast` is off for ranges whose reciprocal is not a normal number.
struct Quantizer {
    float m, delta, rinv, Lf;
    bool fast;
    __device__ __forceinline__ void set(float mg, float L)
    {
        m = mg;
        Lf = L;
        const float hg = (mg == 0.0f) ? 0.0f : __fdiv_rn(mg, L);
        delta = (mg == 0.0f) ? 1.0f : 2.0f * hg;  // all-zero group: w + m = 0 gives code 0 with any Delta
        rinv = __fdiv_rn(1.0f, delta);
        fast = delta >= 1.0e-30f && delta <= 1.0e30f;
    }
    // a general range [lo, lo + L*d] (q0 = lo): code = rint(fl(fl(w - lo) / d)); d = 0 (a constant group) gives
    // code 0 for every w = lo.  For lo <= w <= hi and d = fl(fl(hi - lo)/L) the quotient stays below L + 1/2.
    __device__ __forceinline__ void set_range(float lo, float d)
    {
        m = -lo;
        Lf = 0.0f;
        delta = (d == 0.0f) ? 1.0f : d;
        rinv = __fdiv_rn(1.0f, delta);
        fast = delta >= 1.0e-30f && delta <= 1.0e30f;
    }
    __device__ __forceinline__ float half_step() const { return (m == 0.0f) ? 0.0f : __fdiv_rn(m, Lf); }
    // rint((w + m)/Delta) as a float.  No clamp to [0, L] is needed: |w| <= m gives 0 <= s <= 2m(1+2^-24),
    // so 0 <= t <= L(1+2^-23) and rint(t) is already in 0..L (callers clamp activations to [-m, m] first).
    __device__ __forceinline__ float code_f(float w) const
    {
        const float s = __fadd_rn(w, m);
        if (fast) {
            const float tp = __fmul_rn(s, rinv);
            float r = rintf(tp);
            if (!(fabsf(tp - r) <= 0.4999f)) r = rintf(__fdiv_rn(s, delta));  // rare; also catches NaN
            return r;
        }
        return rintf(__fdiv_rn(s, delta));
    }
    __device__ __forceinline__ uint32_t code(float w) const { return (uint32_t)code_f(w); }
    // four codes, one per byte (v_cvt_pk_u8_f32 converts and inserts in one instruction; its input is
    // an integer-valued float here, so its rounding never comes into play).  FAST (the caller has tested `fast`
    // once for the range): the reciprocal route for all four and one test for the lot: if any of the four products
    // came within 1e-4 of a rounding boundary, all four are redone with the division (for the other three it gives
    // the same code, by the bound above).  One branch per four weights instead of one per weight.
    template <bool FAST>
    __device__ __forceinline__ uint32_t code4t(const float4 v) const
    {
        if constexpr (FAST) {
            // one weight at a time, so that few values are alive at once (the callers hold whole groups in registers)
            float t = __fmul_rn(__fadd_rn(v.x, m), rinv), r = rintf(t);
            float far = fabsf(t - r);
            uint32_t q = __builtin_amdgcn_cvt_pk_u8_f32(r, 0, 0u);
            t = __fmul_rn(__fadd_rn(v.y, m), rinv); r = rintf(t);
            far = fmaxf(far, fabsf(t - r));
            q = __builtin_amdgcn_cvt_pk_u8_f32(r, 1, q);
            t = __fmul_rn(__fadd_rn(v.z, m), rinv); r = rintf(t);
            far = fmaxf(far, fabsf(t - r));
            q = __builtin_amdgcn_cvt_pk_u8_f32(r, 2, q);
            t = __fmul_rn(__fadd_rn(v.w, m), rinv); r = rintf(t);
            far = fmaxf(far, fabsf(t - r));
            q = __builtin_amdgcn_cvt_pk_u8_f32(r, 3, q);
            if (far <= 0.4999f) return q;  // (false also for NaN)
        }
        uint32_t q = __builtin_amdgcn_cvt_pk_u8_f32(rintf(__fdiv_rn(__fadd_rn(v.x, m), delta)), 0, 0u);
        q = __builtin_amdgcn_cvt_pk_u8_f32(rintf(__fdiv_rn(__fadd_rn(v.y, m), delta)), 1, q);
        q = __builtin_amdgcn_cvt_pk_u8_f32(rintf(__fdiv_rn(__fadd_rn(v.z, m), delta)), 2, q);
        q = __builtin_amdgcn_cvt_pk_u8_f32(rintf(__fdiv_rn(__fadd_rn(v.w, m), delta)), 3, q);
        return q;
    }
    __device__ __forceinline__ uint32_t code4(const float4 v) const { return fast ? code4t<true>(v) : code4t<false>(v); }
};

// ---- host-side argument checks ------------------------------------------------------------------
inline bool bits_ok(int bits) { return bits == 2 || bits == 3 || bits == 4 || bits == 8; }
inline bool k_ok(int64_t K) { return K > 0 && K % QB_K_ALIGN == 0 && K <= QB_MAX_K; }
inline qb_status launch_status() { return hipGetLastError() == hipSuccess ? QB_OK : QB_ERR_HIP; }

}  // namespace qb
