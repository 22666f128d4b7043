// Streaming kernels: bf16 -> block-scaled FP8/FP4 quantization (SNIP Sec. 2.3, applied to
// the tensors Sec. 2.2 names) and the quantization-error statistics of Sec. 3.1 Step 1
// (row-wise form: Sec. 5.3).  All of them are bound by HBM bandwidth: one 2-byte read per
// element, 0.53 / 1.03 bytes written (FP4 / FP8), and a handful of VALU ops per element.
//
// A block of 32 elements is handled as follows.
//   amax    : integer maximum of the bf16 magnitude bits (order-preserving for non-negative
//             floats), packed 2 x u16 per VGPR.
//   scale   : integer function of amax's exponent and mantissa fields (no log2).
//   cast    : gfx950's v_cvt_scalef32_pk_{fp8,fp4}_bf16, which divides by the power of two
//             in the scale operand's exponent field and rounds to nearest even.  The FP4
//             form saturates; the FP8 form does not, so under the floor rule magnitudes are
//             clamped to 448 * 2^e first (the no-overflow rule never exceeds it).
//   error   : v_cvt_scalef32_pk_f32_{fp8,fp4} gives q(x) exactly in fp32; the difference to x
//             (exact in fp32) is squared and summed in fp32 per lane, then per wave, and the
//             per-wave partials are summed in double by a single-block kernel in fixed order.
#include "snip_internal.h"
#include <cstdlib>

namespace snip {
namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

template <int FMT> struct Fmt;
template <> struct Fmt<kFP8> { static constexpr int emax = 8; static constexpr unsigned mmax = 0x60; };  // 448 = 1.75 * 2^8
template <> struct Fmt<kFP4> { static constexpr int emax = 2; static constexpr unsigned mmax = 0x40; };  // 6   = 1.5  * 2^2

// Source loads.  A source line is read once and never again, so its load carries the streaming hint (measured:
// quantize ROW 4.7 -> 5.8 TB/s, COL 4.0 -> 4.75 TB/s of algorithmic bytes on a 361 MB tensor).  The one-pass kernel
// for both orientations reads every line twice, the second time out of cache: both of its reads are plain loads
// (with the hint on either one the kernel got 4-6 % slower).
typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld16(const uint16_t* p)
{
    const v4u_t v = __builtin_nontemporal_load(reinterpret_cast<const v4u_t*>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}
template <bool LAST_USE = true>
__device__ __forceinline__ unsigned ld4(const uint16_t* p)
{
    if (LAST_USE) return __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(p));
    return *reinterpret_cast<const unsigned*>(p);
}

__device__ __forceinline__ unsigned pk_max_u16(unsigned a, unsigned b)
{
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a),
                                                                  __builtin_bit_cast(ushort2_t, b)));
}
__device__ __forceinline__ unsigned pk_min_u16(unsigned a, unsigned b)
{
    return __builtin_bit_cast(unsigned, __builtin_elementwise_min(__builtin_bit_cast(ushort2_t, a),
                                                                  __builtin_bit_cast(ushort2_t, b)));
}

// Maximum over the four lanes of a quad (DPP quad_perm [1,0,3,2] then [2,3,0,1]).
__device__ __forceinline__ unsigned quad_max(unsigned m)
{
    unsigned t = (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, 0xB1, 0xF, 0xF, true);
    m = m > t ? m : t;
    t = (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, 0x4E, 0xF, 0xF, true);
    return m > t ? m : t;
}

__device__ __forceinline__ float wave_sum(float v)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// E8M0 byte from the 15 magnitude bits of the block maximum; 0xFF for Inf/NaN.
template <int FMT, int RULE>
__device__ __forceinline__ unsigned scale_byte(unsigned amax_bits)
{
    int b = (int)(amax_bits >> 7) - Fmt<FMT>::emax;
    if (RULE == 0 && (amax_bits & 0x7Fu) > Fmt<FMT>::mmax) b += 1;
    b = b < 0 ? 0 : b;
    return amax_bits >= 0x7F80u ? 0xFFu : (unsigned)b;
}

// The conversion instructions read only the exponent field of their scale operand; the
// mantissa bit set here keeps byte 0 (2^-127) from being an all-zero word.
__device__ __forceinline__ float scale_operand(unsigned byte)
{
    return __uint_as_float((byte << 23) | 0x00400000u);
}

// Clamp both bf16 halves of w to magnitude <= 448 * 2^(byte-127) (floor rule, FP8 only).
__device__ __forceinline__ unsigned clamp_fp8(unsigned w, unsigned byte)
{
    const unsigned lim = ((byte + 8u) << 7) | 0x60u;
    const unsigned mag = pk_min_u16(w & 0x7FFF7FFFu, lim | (lim << 16));
    return mag | (w & 0x80008000u);
}

// A register with unspecified content, at no cost: the packing conversions below replace their destination piece by
// piece (two halves for FP8, four bytes for FP4) and keep the rest, so the value they start from never survives;
// starting from zero would cost a move per destination.
__device__ __forceinline__ unsigned any_value()
{
    unsigned r;
    asm volatile("" : "=v"(r));
    return r;
}

// Two bf16 pairs (4 elements) -> 4 FP8 bytes.
template <int RULE>
__device__ __forceinline__ unsigned enc8(unsigned w0, unsigned w1, float sc, unsigned byte)
{
    if (RULE == 1) { w0 = clamp_fp8(w0, byte); w1 = clamp_fp8(w1, byte); }
    short2_t r = __builtin_bit_cast(short2_t, any_value());
    r = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(r, __builtin_bit_cast(bf16x2, w0), sc, false);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(r, __builtin_bit_cast(bf16x2, w1), sc, true);
    return __builtin_bit_cast(unsigned, r);
}

// Four bf16 pairs (8 elements) -> 8 FP4 nibbles, element 0 in the lowest nibble.
__device__ __forceinline__ unsigned enc4(unsigned w0, unsigned w1, unsigned w2, unsigned w3, float sc)
{
    unsigned r = any_value();
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(r, __builtin_bit_cast(bf16x2, w0), sc, 0);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(r, __builtin_bit_cast(bf16x2, w1), sc, 1);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(r, __builtin_bit_cast(bf16x2, w2), sc, 2);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(r, __builtin_bit_cast(bf16x2, w3), sc, 3);
    return r;
}

// ---- stochastic rounding to FP4 (Sec. 5.1: FP4 output gradients are rounded probabilistically to the two
//      nearest values).  Definition: with lo <= |v| <= hi the neighbouring grid magnitudes of the scaled
//      element and p = (|v| - lo) / (hi - lo), the magnitude goes up iff rnd < floor(256 p), rnd being the
//      element's random byte: byte (i mod 8) of Threefry-2x32-20(counter = i div 8, key = seed), i the
//      element's row-major position in the stored matrix. ----

// Threefry-2x32, 20 rounds (Salmon et al., SC'11): adds, rotates and XORs only, which suits a VALU whose
// 32-bit multiplies run at quarter rate.
__device__ __forceinline__ unsigned rotl32(unsigned v, int r) { return (v << r) | (v >> (32 - r)); }
__device__ __forceinline__ void threefry2x32_20(unsigned c0, unsigned c1, unsigned k0, unsigned k1,
                                                unsigned& o0, unsigned& o1)
{
    constexpr int R[8] = {13, 15, 26, 6, 17, 29, 16, 24};
    const unsigned ks[3] = {k0, k1, 0x1BD11BDAu ^ k0 ^ k1};
    unsigned x0 = c0 + ks[0], x1 = c1 + ks[1];
#pragma unroll
    for (int r = 0; r < 20; ++r) {
        x0 += x1;
        x1 = rotl32(x1, R[r % 8]) ^ x0;
        if (r % 4 == 3) {
            const int inj = r / 4 + 1;
            x0 += ks[inj % 3];
            x1 += ks[(inj + 1) % 3] + (unsigned)inj;
        }
    }
    o0 = x0; o1 = x1;
}

// The rule is carried out by gfx950's stochastic-rounding conversion v_cvt_scalef32_sr_pk_fp4_f32.  What that
// instruction does was established on the hardware for every bf16 magnitude from 2^-12 to 6 (both signs)
// against 256 seeds per operand slot: for the first element of its pair it adds bits [31:10] of the seed
// to the 22 mantissa bits that FP4 drops (denormalised below 1) and rounds up on a carry, so with a seed
// R << 24 it rounds up iff floor(256 p) + R >= 256 -- the rule above with R = 255 - rnd.  The second
// element of a pair takes the seed shifted by one bit, which would tie its random number to the first
// one's; every element therefore goes through the first slot of its own instruction (second slot 0.0).
// Bits below the top eight of the seed must be zero, or they could carry into the comparison.
// The instruction is written as inline assembly: it replaces one byte of its destination and keeps the
// other three, and the compiler's builtin for it does not tie the destination to the previous value.
typedef float float2_t_sr __attribute__((ext_vector_type(2)));
#define SNIP_SR_CVT(dst, src, seed, sc, OPSEL) \
    asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, %3" OPSEL : "+v"(dst) : "v"(src), "v"(seed), "v"(sc))

// Four bf16 pairs (8 consecutive stored elements) -> 8 FP4 nibbles with stochastic rounding; r0 holds
// the random bytes of elements 0-3, r1 those of elements 4-7; sc is the block scale operand.
__device__ __forceinline__ unsigned enc4_sr(const unsigned* w, float sc, unsigned r0, unsigned r1)
{
    const unsigned n0 = ~r0, n1 = ~r1;                      // 255 - rnd in every byte
    unsigned even = 0, odd = 0;                             // byte i: code of element 2i / 2i+1 in its low nibble
    float2_t_sr xe[4], xo[4];
    unsigned se[4], so[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const unsigned nn = i < 2 ? n0 : n1;
        // byte (2i mod 4) resp. (2i+1 mod 4) of nn moved to the top byte, zeros below
        se[i] = __builtin_amdgcn_perm(nn, 0u, (i & 1) ? 0x060C0C0Cu : 0x040C0C0Cu);
        so[i] = __builtin_amdgcn_perm(nn, 0u, (i & 1) ? 0x070C0C0Cu : 0x050C0C0Cu);
        xe[i] = float2_t_sr{__uint_as_float(w[i] << 16), 0.f};
        xo[i] = float2_t_sr{__uint_as_float(w[i] & 0xFFFF0000u), 0.f};
    }
    SNIP_SR_CVT(even, xe[0], se[0], sc, "");
    SNIP_SR_CVT(even, xe[1], se[1], sc, " op_sel:[0,0,1,0]");
    SNIP_SR_CVT(even, xe[2], se[2], sc, " op_sel:[0,0,0,1]");
    SNIP_SR_CVT(even, xe[3], se[3], sc, " op_sel:[0,0,1,1]");
    SNIP_SR_CVT(odd, xo[0], so[0], sc, "");
    SNIP_SR_CVT(odd, xo[1], so[1], sc, " op_sel:[0,0,1,0]");
    SNIP_SR_CVT(odd, xo[2], so[2], sc, " op_sel:[0,0,0,1]");
    SNIP_SR_CVT(odd, xo[3], so[3], sc, " op_sel:[0,0,1,1]");
    return even | (odd << 4);
}
#undef SNIP_SR_CVT

// Codes of the 8 consecutive stored elements that start at stored position e0 (a multiple of 8).
__device__ __forceinline__ unsigned enc4_sr_at(const unsigned* w, float sc, int64_t e0, uint2 seed)
{
    const uint64_t grp = (uint64_t)e0 >> 3;
    unsigned r0, r1;
    threefry2x32_20((unsigned)grp, (unsigned)(grp >> 32), seed.x, seed.y, r0, r1);
    return enc4_sr(w, sc, r0, r1);
}

// s0 += x_lo^2 + x_hi^2 for a bf16 pair (one instruction: the products are exact, the sum is rounded once)
__device__ __forceinline__ void acc_sq(unsigned w, float& s0)
{
    asm("v_dot2c_f32_bf16 %0, %1, %1" : "+v"(s0) : "v"(w));
}
__device__ __forceinline__ void acc_err(float2_t q, unsigned w, float& s0, float& se, bool want_s0)
{
    const float xl = __uint_as_float(w << 16), xh = __uint_as_float(w & 0xFFFF0000u);
    const float dl = q[0] - xl, dh = q[1] - xh;
    se = fmaf(dl, dl, se);
    se = fmaf(dh, dh, se);
    if (want_s0) acc_sq(w, s0);
}

// Error sums of 8 source elements w[0..3] against their FP8 codes c[0..1].
__device__ __forceinline__ void err8(const unsigned* w, unsigned c0, unsigned c1, float sc,
                                     float& s0, float& se, bool want_s0)
{
    acc_err(__builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c0, sc, false), w[0], s0, se, want_s0);
    acc_err(__builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c0, sc, true),  w[1], s0, se, want_s0);
    acc_err(__builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c1, sc, false), w[2], s0, se, want_s0);
    acc_err(__builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c1, sc, true),  w[3], s0, se, want_s0);
}
__device__ __forceinline__ void err4(const unsigned* w, unsigned c, float sc,
                                     float& s0, float& se, bool want_s0)
{
    acc_err(__builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c, sc, 0), w[0], s0, se, want_s0);
    acc_err(__builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c, sc, 1), w[1], s0, se, want_s0);
    acc_err(__builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c, sc, 2), w[2], s0, se, want_s0);
    acc_err(__builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c, sc, 3), w[3], s0, se, want_s0);
}

// Magnitude bits of the largest of the 8 bf16 values in v (one lane's share of a block).
__device__ __forceinline__ unsigned amax8(const uint4& v)
{
    unsigned m = pk_max_u16(pk_max_u16(v.x & 0x7FFF7FFFu, v.y & 0x7FFF7FFFu),
                            pk_max_u16(v.z & 0x7FFF7FFFu, v.w & 0x7FFF7FFFu));
    const unsigned lo = m & 0xFFFFu, hi = m >> 16;
    return lo > hi ? lo : hi;
}

// ------------------------------------------------------------------------------------------
// Row blocks.  A lane owns 8 consecutive elements (one 16-byte load), a quad owns a block, a
// wave owns 512 consecutive elements of a row ("segment").  Four segments are in flight per
// wave.  Loads and code stores are fully coalesced; the 16 scale bytes of a segment are
// written by the first lane of each quad to 16 consecutive addresses.
// ------------------------------------------------------------------------------------------
constexpr int kSeg = 512;
constexpr int kUnroll = 4;
constexpr int kStatUnroll = 8;         // loads in flight per lane in the row statistics kernel

template <int FMT, int RULE, bool STATS, bool SR = false>
__global__ __launch_bounds__(256) void quant_row_kernel(const uint16_t* __restrict__ x, int rows,
                                                        int cols, int64_t ld,
                                                        uint8_t* __restrict__ codes,
                                                        uint8_t* __restrict__ scales,
                                                        uint8_t* __restrict__ scales_g4, int64_t kpitch,
                                                        float* __restrict__ partials, uint2 seed)
{
    static_assert(!SR || (FMT == kFP4 && !STATS), "stochastic rounding: FP4, no fused statistics");
    // unit = (group of 4 consecutive rows, 512-element segment); the wave's four loads in flight
    // are the four rows, so that the block-major scale copy gets one dword (4 rows) per block.
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    const int nwaves = gridDim.x * kWavesPerBlock;
    const int spr = (cols + kSeg - 1) / kSeg;
    const int units = ((rows + kUnroll - 1) / kUnroll) * spr;
    const int nblk = cols / kBlock;
    float s0 = 0.f, se = 0.f;

    for (int u = wave; u < units; u += nwaves) {
        const int rg = u / spr;
        const int col = (u - rg * spr) * kSeg + lane * 8;
        uint4 v[kUnroll];
        bool act[kUnroll];
#pragma unroll
        for (int j = 0; j < kUnroll; ++j) {
            const int row = rg * kUnroll + j;
            act[j] = row < rows && col < cols;
            v[j] = make_uint4(0, 0, 0, 0);
            if (act[j]) v[j] = ld16(x + (int64_t)row * ld + col);
        }
        unsigned packed = 0;
#pragma unroll
        for (int j = 0; j < kUnroll; ++j) {
            const int row = rg * kUnroll + j;
            const unsigned am = quad_max(amax8(v[j]));
            const unsigned byte = scale_byte<FMT, RULE>(am);
            const float sc = scale_operand(byte);
            const bool bad = byte == 0xFFu;
            const unsigned w[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
            const int64_t e0 = (int64_t)row * cols + col;
            if (FMT == kFP8) {
                unsigned c0 = enc8<RULE>(w[0], w[1], sc, byte), c1 = enc8<RULE>(w[2], w[3], sc, byte);
                if (bad) { c0 = 0; c1 = 0; }
                if (act[j]) *reinterpret_cast<uint2*>(codes + e0) = make_uint2(c0, c1);
                if (STATS) err8(w, c0, c1, sc, s0, se, true);
            } else {
                unsigned c = SR ? enc4_sr_at(w, sc, e0, seed) : enc4(w[0], w[1], w[2], w[3], sc);
                if (bad) c = 0;
                if (act[j]) *reinterpret_cast<unsigned*>(codes + (e0 >> 1)) = c;
                if (STATS) err4(w, c, sc, s0, se, true);
            }
            if (act[j] && (lane & 3) == 0)
                scales[(int64_t)row * nblk + (col >> 5)] = (uint8_t)byte;
            packed |= byte << (8 * j);
        }
        // Grouped copy: `packed` holds this block's byte for each of the 4 rows.  Fetch the same
        // word from the next three quads (the next three blocks of the same 128-element group),
        // transpose the 4x4 bytes, and let the first lane of every 16 store the four rows' dwords
        // (16 contiguous bytes).  Rows past the end fall inside the padded pitch.
        if (scales_g4) {
            const unsigned p0 = packed;
            const unsigned p1 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)packed, 0x104, 0xF, 0xF, true);   // lane + 4
            const unsigned p2 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)packed, 0x108, 0xF, 0xF, true);   // lane + 8
            const unsigned p3 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)packed, 0x10C, 0xF, 0xF, true);   // lane + 12
            const unsigned a_lo = __builtin_amdgcn_perm(p1, p0, 0x05010400u), a_hi = __builtin_amdgcn_perm(p1, p0, 0x07030602u);
            const unsigned b_lo = __builtin_amdgcn_perm(p3, p2, 0x05010400u), b_hi = __builtin_amdgcn_perm(p3, p2, 0x07030602u);
            const uint4 d = make_uint4(__builtin_amdgcn_perm(b_lo, a_lo, 0x05040100u), __builtin_amdgcn_perm(b_lo, a_lo, 0x07060302u),
                                       __builtin_amdgcn_perm(b_hi, a_hi, 0x05040100u), __builtin_amdgcn_perm(b_hi, a_hi, 0x07060302u));
            if (col < cols && (lane & 15) == 0)
                *reinterpret_cast<uint4*>(scales_g4 + ((int64_t)(col >> 7) * kpitch + rg * kUnroll) * 4) = d;
        }
    }
    if (STATS) {
        s0 = wave_sum(s0);
        se = wave_sum(se);
        if (lane == 0) { partials[wave * 3 + 0] = s0; partials[wave * 3 + 1] = se; partials[wave * 3 + 2] = 0.f; }
    }
}

// Statistics only, both formats, row blocks.  One wave walks whole rows so that the per-row
// sums of Sec. 5.3 come out of the same pass.
template <int RULE>
__global__ __launch_bounds__(256) void stats_row_kernel(const uint16_t* __restrict__ x, int rows,
                                                        int cols, int64_t ld,
                                                        float* __restrict__ partials,
                                                        float* __restrict__ per_line)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    const int nwaves = gridDim.x * kWavesPerBlock;
    float t0 = 0.f, t4 = 0.f, t8 = 0.f;
    for (int row = wave; row < rows; row += nwaves) {
        const uint16_t* xr = x + (int64_t)row * ld;
        float s0 = 0.f, s4 = 0.f, s8 = 0.f;
        for (int c0 = 0; c0 < cols; c0 += kSeg * kStatUnroll) {
            uint4 v[kStatUnroll];
#pragma unroll
            for (int j = 0; j < kStatUnroll; ++j) {
                const int col = c0 + j * kSeg + lane * 8;
                v[j] = make_uint4(0, 0, 0, 0);     // zeros quantize to zero: no contribution
                if (col < cols) v[j] = ld16(xr + col);
            }
#pragma unroll
            for (int j = 0; j < kStatUnroll; ++j) {
                if (c0 + j * kSeg >= cols) break;                    // wave-uniform: the row has no such segment
                const unsigned am = quad_max(amax8(v[j]));
                const unsigned b8 = scale_byte<kFP8, RULE>(am), b4 = scale_byte<kFP4, RULE>(am);
                const float sc8 = scale_operand(b8), sc4 = scale_operand(b4);
                const unsigned w[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
                const unsigned c0_ = enc8<RULE>(w[0], w[1], sc8, b8), c1_ = enc8<RULE>(w[2], w[3], sc8, b8);
                const unsigned c4 = enc4(w[0], w[1], w[2], w[3], sc4);
                float dummy = 0.f;
                err8(w, c0_, c1_, sc8, s0, s8, true);
                err4(w, c4, sc4, dummy, s4, false);
                if (b8 == 0xFFu) { s4 = __builtin_nanf(""); s8 = __builtin_nanf(""); }
            }
        }
        s0 = wave_sum(s0); s4 = wave_sum(s4); s8 = wave_sum(s8);
        if (per_line && lane == 0) {
            per_line[(int64_t)row * 3 + 0] = s0; per_line[(int64_t)row * 3 + 1] = s4; per_line[(int64_t)row * 3 + 2] = s8;
        }
        t0 += s0; t4 += s4; t8 += s8;
    }
    if (lane == 0) { partials[wave * 3 + 0] = t0; partials[wave * 3 + 1] = t4; partials[wave * 3 + 2] = t8; }
}

// ------------------------------------------------------------------------------------------
// Column blocks.  A lane owns two adjacent columns and reads them one dword per row: a wave
// reads 256 contiguous bytes of each of 32 rows (one block per column), 32 independent loads
// in flight.  The block maximum of a column never leaves the lane.  Rows are re-paired with
// v_perm so that the conversion instructions pack elements that are adjacent in the
// transposed output; each lane then stores 32 (FP8) or 16 (FP4) contiguous bytes per column.
// A wave processes four (FP8) or eight (FP4) vertically adjacent blocks back to back, i.e. exactly one
// 128-byte line of every stored row, so that no line of the output is written in two pieces.
// ------------------------------------------------------------------------------------------
constexpr int kColsPerWave = 128;
constexpr int kRowBlocksPerUnit = 4;

struct ColBlock {
    unsigned lo[16], hi[16];   // bf16 pairs (row 2k, row 2k+1) of the lane's two columns
    unsigned am_lo, am_hi;     // magnitude bits of each column's block maximum
};

// (the caller reads these lines again)
__device__ __forceinline__ void load_col_raw(const uint16_t* __restrict__ p, int64_t ld, unsigned (&v)[32])
{
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = ld4<false>(p + (int64_t)i * ld);
}

__device__ __forceinline__ void pair_col_block(const unsigned (&v)[32], ColBlock& b)
{
    unsigned m = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) m = pk_max_u16(m, v[i] & 0x7FFF7FFFu);
    b.am_lo = m & 0xFFFFu;
    b.am_hi = m >> 16;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        b.lo[k] = __builtin_amdgcn_perm(v[2 * k + 1], v[2 * k], 0x05040100u);
        b.hi[k] = __builtin_amdgcn_perm(v[2 * k + 1], v[2 * k], 0x07060302u);
    }
}

__device__ __forceinline__ void load_col_block(const uint16_t* __restrict__ p, int64_t ld, bool act, ColBlock& b)
{
    unsigned v[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = act ? ld4(p + (int64_t)i * ld) : 0u;
    unsigned m = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) m = pk_max_u16(m, v[i] & 0x7FFF7FFFu);
    b.am_lo = m & 0xFFFFu;
    b.am_hi = m >> 16;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        b.lo[k] = __builtin_amdgcn_perm(v[2 * k + 1], v[2 * k], 0x05040100u);
        b.hi[k] = __builtin_amdgcn_perm(v[2 * k + 1], v[2 * k], 0x07060302u);
    }
}

// Codes of one column's block (32 rows) -> the wave's LDS staging area; returns the scale byte.
// In LDS the wave keeps a [128 stored rows][ROWB bytes] image of its unit's output (ROWB = 128: 128 source
// rows of FP8 codes or 256 of FP4 codes); 16-byte chunk c of row r sits at position c ^ ((r >> 1) & (CPR-1)).
template <int FMT, int RULE, bool STATS, bool SR>
__device__ __forceinline__ unsigned quant_one_column(const unsigned* w, unsigned am, uint8_t* __restrict__ lds_row,
                                                     int rb_local, int swz, float& s0, float& se,
                                                     int64_t e0, uint2 seed)      // e0: stored position of w[0]'s first element
{
    const unsigned byte = scale_byte<FMT, RULE>(am);
    const float sc = scale_operand(byte);
    const bool bad = byte == 0xFFu;
    if (FMT == kFP8) {
        unsigned c[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            c[k] = enc8<RULE>(w[2 * k], w[2 * k + 1], sc, byte);
            if (bad) c[k] = 0;
        }
        *reinterpret_cast<uint4*>(lds_row + (((rb_local * 2 + 0) ^ swz) * 16)) = make_uint4(c[0], c[1], c[2], c[3]);
        *reinterpret_cast<uint4*>(lds_row + (((rb_local * 2 + 1) ^ swz) * 16)) = make_uint4(c[4], c[5], c[6], c[7]);
        if (STATS) {
#pragma unroll
            for (int k = 0; k < 4; ++k) err8(w + 4 * k, c[2 * k], c[2 * k + 1], sc, s0, se, true);
        }
    } else {
        unsigned c[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            c[k] = SR ? enc4_sr_at(w + 4 * k, sc, e0 + 8 * k, seed)
                      : enc4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3], sc);
            if (bad) c[k] = 0;
        }
        *reinterpret_cast<uint4*>(lds_row + ((rb_local ^ swz) * 16)) = make_uint4(c[0], c[1], c[2], c[3]);
        if (STATS) {
#pragma unroll
            for (int k = 0; k < 4; ++k) err4(w + 4 * k, c[k], sc, s0, se, true);
        }
    }
    return byte;
}

// COOP: the four waves of a workgroup share one unit (wave w takes its row blocks w, w + 4) and one staging area, so
// that a workgroup needs 17 KB of LDS instead of 64 KB and more waves are resident; the scale bytes of the four row
// blocks of a dword meet in LDS.  Same bytes out.
template <int FMT, int RULE, bool STATS, bool SR = false, bool COOP = false>
__global__ __launch_bounds__(256) void quant_col_kernel(const uint16_t* __restrict__ x, int rows,
                                                        int cols, int64_t ld,
                                                        uint8_t* __restrict__ codes,
                                                        uint8_t* __restrict__ scales,
                                                        uint8_t* __restrict__ scales_g4, int64_t kpitch,
                                                        float* __restrict__ partials, uint2 seed)
{
    static_assert(!SR || (FMT == kFP4 && !STATS), "stochastic rounding: FP4, no fused statistics");
    // row blocks per unit: one full 128-byte line of every stored row (128 FP8 / 256 FP4 source rows); the
    // stochastic variant, bound by VALU work and register count rather than by stores, keeps half lines
    constexpr int RBU = FMT == kFP8 ? 4 : (SR ? 4 : 8);
    constexpr int ROWB = RBU * (FMT == kFP8 ? 32 : 16);   // staged output bytes per stored row
    constexpr int CPR = ROWB / 16;
    __shared__ __attribute__((aligned(16))) uint8_t stage[COOP ? 1 : kWavesPerBlock][kColsPerWave * ROWB];
    __shared__ __attribute__((aligned(4))) uint8_t scale_stage[COOP ? RBU * kColsPerWave : 4];   // COOP: scale byte of (row block, column)
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint8_t* const reg = stage[COOP ? 0 : wib];
    const int wave = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + wib);
    const int nwaves = gridDim.x * kWavesPerBlock;
    const int ncg = (cols + kColsPerWave - 1) / kColsPerWave;
    const int nrb = rows / kBlock;
    const int nru = (nrb + RBU - 1) / RBU;
    const int units = ncg * nru;
    const int64_t out_row_bytes = FMT == kFP8 ? rows : rows / 2;
    float s0 = 0.f, se = 0.f;
    for (int u = COOP ? (int)blockIdx.x : wave; u < units; u += COOP ? (int)gridDim.x : nwaves) {
        const int ru = u / ncg, cg = u - ru * ncg;
        const int c = cg * kColsPerWave + lane * 2;
        const bool act = c < cols;
        const int rb0 = ru * RBU;
        const int nb = min(nrb - rb0, RBU);
        const int swz_lo = lane & (CPR - 1);          // ((2 * lane) >> 1) & (CPR - 1); the odd row shares it
        // row block kk of the unit: codes into the staging area, returns the two columns' scale bytes
        auto one_block = [&](int kk, unsigned& y0, unsigned& y1) {
            ColBlock b;
            load_col_block(x + (int64_t)(rb0 + kk) * kBlock * ld + c, ld, act, b);
            const int64_t e0 = (int64_t)c * rows + (int64_t)(rb0 + kk) * kBlock;       // stored row = source column
            y0 = quant_one_column<FMT, RULE, STATS, SR>(b.lo, b.am_lo, reg + (2 * lane) * ROWB, kk, swz_lo, s0, se, e0, seed);
            y1 = quant_one_column<FMT, RULE, STATS, SR>(b.hi, b.am_hi, reg + (2 * lane + 1) * ROWB, kk, swz_lo, s0, se, e0 + rows, seed);
        };
        // Four row blocks at a time (blocks 0 .. last of the group starting at rbh): their scale bytes of a column
        // form one dword of the row-major array (when the row length allows it) and exactly one dword of the
        // grouped copy.
        auto store_scales = [&](int rbh, int last, unsigned lo, unsigned hi) {
            if (act) {
                uint8_t* s_lo = scales + (int64_t)c * nrb + rbh;
                if ((nrb & 3) == 0) {
                    *reinterpret_cast<unsigned*>(s_lo) = lo;
                    *reinterpret_cast<unsigned*>(s_lo + nrb) = hi;
                } else {
                    for (int k = 0; k <= last; ++k) { s_lo[k] = (uint8_t)(lo >> (8 * k)); s_lo[nrb + k] = (uint8_t)(hi >> (8 * k)); }
                }
                if (scales_g4)
                    *reinterpret_cast<uint2*>(scales_g4 + ((int64_t)(rbh / kRowBlocksPerUnit) * kpitch + c) * 4) = make_uint2(lo, hi);
            }
        };
        if (COOP) {
            for (int kk = wib; kk < nb; kk += kWavesPerBlock) {
                unsigned y0, y1;
                one_block(kk, y0, y1);
                *reinterpret_cast<uint16_t*>(scale_stage + kk * kColsPerWave + 2 * lane) = (uint16_t)(y0 | (y1 << 8));
            }
            __syncthreads();                                   // all row blocks of the unit are staged
            for (int h = wib; h * kRowBlocksPerUnit < nb; h += kWavesPerBlock) {
                const int last = min(kRowBlocksPerUnit - 1, nb - 1 - h * kRowBlocksPerUnit);
                unsigned lo = 0, hi = 0;
                for (int k = 0; k <= last; ++k) {
                    const unsigned v = *reinterpret_cast<const uint16_t*>(scale_stage + (h * kRowBlocksPerUnit + k) * kColsPerWave + 2 * lane);
                    lo |= (v & 0xFFu) << (8 * k);
                    hi |= (v >> 8) << (8 * k);
                }
                store_scales(rb0 + h * kRowBlocksPerUnit, last, lo, hi);
            }
        } else {
            for (int h = 0; h < RBU / kRowBlocksPerUnit; ++h) {
                const int nbh = min(nb - h * kRowBlocksPerUnit, kRowBlocksPerUnit);
                if (nbh <= 0) break;
                unsigned g4_lo = 0, g4_hi = 0;
                for (int k = 0; k < nbh; ++k) {
                    unsigned y0, y1;
                    one_block(h * kRowBlocksPerUnit + k, y0, y1);
                    g4_lo |= y0 << (8 * k);
                    g4_hi |= y1 << (8 * k);
                }
                store_scales(rb0 + h * kRowBlocksPerUnit, nbh - 1, g4_lo, g4_hi);
            }
        }
        // Codes: read the staged image back row-contiguous and store 16 bytes per lane, so that every store
        // instruction writes whole ROWB-byte runs of 64 / CPR stored rows.
#pragma unroll
        for (int it = COOP ? wib : 0; it < kColsPerWave * CPR / 64; it += COOP ? kWavesPerBlock : 1) {
            const int idx = it * 64 + lane;
            const int row = idx / CPR, chunk = idx % CPR;
            const uint4 v = *reinterpret_cast<const uint4*>(reg + row * ROWB + ((chunk ^ ((row >> 1) & (CPR - 1))) * 16));
            const int cc = cg * kColsPerWave + row;
            const int blk = FMT == kFP8 ? chunk >> 1 : chunk;        // row block this chunk belongs to
            if (cc < cols && blk < nb)
                *reinterpret_cast<uint4*>(codes + (int64_t)cc * out_row_bytes + (int64_t)ru * ROWB + chunk * 16) = v;
        }
        if (COOP) __syncthreads();                             // the staging areas go to the next unit
    }
    if (STATS) {
        s0 = wave_sum(s0);
        se = wave_sum(se);
        if (lane == 0) { partials[wave * 3 + 0] = s0; partials[wave * 3 + 1] = se; partials[wave * 3 + 2] = 0.f; }
    }
}

// Both orientations of one tensor from one pass over HBM (Sec. 2.2: X feeds the forward GEMM with blocks along
// its rows and the weight-gradient GEMM with blocks down its columns; W and dY likewise).  A wave owns the same
// units as in quant_col_kernel.  For each 32-row x 128-column tile it runs the column-block path above and then
// reads the tile a second time with the row kernel's lane layout (a lane = 8 consecutive elements, a quad = one
// block, 16 lanes = the tile's 128 columns of one row, 4 rows per load): those loads hit in cache, the lines
// having just been fetched by the same wave.  Results are bit-identical to the two single-orientation kernels.
// Error sum of one column's block (w: its 32 elements as 16 bf16 pairs, am: magnitude bits of its maximum) under
// the format that is NOT being written; no codes leave the lane.
template <int FMT, int RULE>
__device__ __forceinline__ void other_format_error(const unsigned* w, unsigned am, float& se)
{
    const unsigned byte = scale_byte<FMT, RULE>(am);
    const float sc = scale_operand(byte);
    float unused = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (FMT == kFP8) err8(w + 4 * k, enc8<RULE>(w[4 * k], w[4 * k + 1], sc, byte), enc8<RULE>(w[4 * k + 2], w[4 * k + 3], sc, byte), sc, unused, se, false);
        else             err4(w + 4 * k, enc4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3], sc), sc, unused, se, false);
    }
}

// COOP: the four waves of a workgroup share one unit (wave w takes its tiles w, w + 4, ...) and one staging area,
// for tensors with too few units to give every SIMD a wave: a unit's tiles are then worked on side by side instead
// of one after the other.  Same bytes out.
template <int FMT_R, int FMT_C, int RULE, int STATS, bool COOP = false>      // STATS: 0 none, 1 the chosen formats' errors, 2 both formats' errors
__global__ __launch_bounds__(256) void quant_both_kernel(const uint16_t* __restrict__ x, int rows, int cols, int64_t ld,
                                                         uint8_t* __restrict__ codes_r, uint8_t* __restrict__ scales_r,
                                                         uint8_t* __restrict__ g4_r, int64_t kpitch_r,
                                                         uint8_t* __restrict__ codes_c, uint8_t* __restrict__ scales_c,
                                                         uint8_t* __restrict__ g4_c, int64_t kpitch_c,
                                                         float* __restrict__ partials)
{
    constexpr int RBU = FMT_C == kFP8 ? 4 : 8;
    constexpr int ROWB = RBU * (FMT_C == kFP8 ? 32 : 16);
    constexpr int CPR = ROWB / 16;
    // Without the statistics the loads of the next tile are issued before the current one is worked on (two sets
    // of 64 registers); with them the wave is bound by its arithmetic and the plain loop is faster.
    constexpr bool PREFETCH = STATS == 0;
    __shared__ __attribute__((aligned(16))) uint8_t stage[COOP ? 1 : kWavesPerBlock][kColsPerWave * ROWB];
    __shared__ __attribute__((aligned(4))) uint8_t scale_stage[COOP ? RBU * kColsPerWave : 4];   // COOP: scale byte of (tile, column)
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint8_t* const reg = stage[COOP ? 0 : wib];
    const int wave = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + wib);
    const int nwaves = gridDim.x * kWavesPerBlock;
    const int ncg = (cols + kColsPerWave - 1) / kColsPerWave;
    const int nrb = rows / kBlock;
    const int nru = (nrb + RBU - 1) / RBU;
    const int units = ncg * nru;
    const int nblk = cols / kBlock;                       // blocks per row of the row-direction output
    constexpr int KSTEP = COOP ? kWavesPerBlock : 1;      // distance between the tiles one wave takes
    const int k_first = COOP ? wib : 0;
    const int64_t out_row_bytes = FMT_C == kFP8 ? rows : rows / 2;
    const uint2 no_seed = make_uint2(0, 0);
    float s0 = 0.f, se_c = 0.f, se_r = 0.f;
    float so_c = 0.f, so_r = 0.f;                         // STATS == 2: error sums of the format not chosen
    for (int u = COOP ? (int)blockIdx.x : wave; u < units; u += COOP ? (int)gridDim.x : nwaves) {
        const int ru = u / ncg, cg = u - ru * ncg;
        const int c = cg * kColsPerWave + lane * 2;
        const bool act = c < cols;
        const int rcol = cg * kColsPerWave + (lane & 15) * 8;       // row direction: this lane's 8 columns
        const bool ract = rcol < cols;
        const int rb0 = ru * RBU;
        const int nb = min(nrb - rb0, RBU);
        const int swz_lo = lane & (CPR - 1);
        // Tiles of the unit, top to bottom.
        unsigned g4_lo = 0, g4_hi = 0;
        // Loads carry no condition (a lane past the last column reads column 0 of the same rows instead and is
        // zeroed afterwards, under a wave-uniform test), so that all 40 of a tile stay in flight together.
        const bool ragged = (cg + 1) * kColsPerWave > cols;
        // Four row blocks done (the last group of a tensor may hold fewer: blocks 0 .. last): their scale bytes of a
        // column are one dword of the row-major array (when the row length allows it) and exactly one dword of the
        // grouped copy.
        auto store_col_scales = [&](int rbh, int last, unsigned lo, unsigned hi) {
            if (act) {
                uint8_t* s_lo = scales_c + (int64_t)c * nrb + rbh;
                if ((nrb & 3) == 0) {
                    *reinterpret_cast<unsigned*>(s_lo) = lo;
                    *reinterpret_cast<unsigned*>(s_lo + nrb) = hi;
                } else {
                    for (int i = 0; i <= last; ++i) { s_lo[i] = (uint8_t)(lo >> (8 * i)); s_lo[nrb + i] = (uint8_t)(hi >> (8 * i)); }
                }
                if (g4_c)
                    *reinterpret_cast<uint2*>(g4_c + ((int64_t)(rbh / kRowBlocksPerUnit) * kpitch_c + c) * 4) = make_uint2(lo, hi);
            }
        };
        auto fetch_row = [&](int k, uint4 (&rv)[8]) {
            const uint16_t* pr = x + (int64_t)((rb0 + k) * kBlock + (lane >> 4)) * ld + (ract ? rcol : 0);
#pragma unroll
            for (int j = 0; j < 8; ++j) rv[j] = *reinterpret_cast<const uint4*>(pr + (int64_t)(4 * j) * ld);
        };
        auto fetch = [&](int k, unsigned (&cv)[32], uint4 (&rv)[8]) {
            load_col_raw(x + (int64_t)(rb0 + k) * kBlock * ld + (act ? c : 0), ld, cv);
            fetch_row(k, rv);
        };
        auto work = [&](int k, unsigned (&cv)[32], uint4 (&rv)[8]) {
            if (ragged) {
#pragma unroll
                for (int i = 0; i < 32; ++i) cv[i] = act ? cv[i] : 0u;
#pragma unroll
                for (int j = 0; j < 8; ++j) rv[j] = ract ? rv[j] : make_uint4(0, 0, 0, 0);
            }
            // ---- column direction
            ColBlock b;
            pair_col_block(cv, b);
            const unsigned y0 = quant_one_column<FMT_C, RULE, STATS != 0, false>(b.lo, b.am_lo, reg + (2 * lane) * ROWB, k, swz_lo, s0, se_c, 0, no_seed);
            const unsigned y1 = quant_one_column<FMT_C, RULE, STATS != 0, false>(b.hi, b.am_hi, reg + (2 * lane + 1) * ROWB, k, swz_lo, s0, se_c, 0, no_seed);
            if (STATS == 2) {
                other_format_error<1 - FMT_C, RULE>(b.lo, b.am_lo, so_c);
                other_format_error<1 - FMT_C, RULE>(b.hi, b.am_hi, so_c);
            }
            if (COOP) {
                // the four tiles of a dword belong to four waves: the bytes meet in LDS after the unit's barrier
                *reinterpret_cast<uint16_t*>(scale_stage + k * kColsPerWave + 2 * lane) = (uint16_t)(y0 | (y1 << 8));
            } else {
                g4_lo |= y0 << (8 * (k & 3));
                g4_hi |= y1 << (8 * (k & 3));
                if ((k & 3) == 3 || k == nb - 1) {
                    store_col_scales(rb0 + (k & ~3), k & 3, g4_lo, g4_hi);
                    g4_lo = 0; g4_hi = 0;
                }
            }
            // ---- row direction
            const int row0 = (rb0 + k) * kBlock + (lane >> 4);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int row = row0 + 4 * j;
                const unsigned am = quad_max(amax8(rv[j]));
                const unsigned byte = scale_byte<FMT_R, RULE>(am);
                const float sc = scale_operand(byte);
                const bool bad = byte == 0xFFu;
                const unsigned w[4] = {rv[j].x, rv[j].y, rv[j].z, rv[j].w};
                const int64_t e0 = (int64_t)row * cols + rcol;
                float unused = 0.f;
                if (FMT_R == kFP8) {
                    unsigned c0 = enc8<RULE>(w[0], w[1], sc, byte), c1 = enc8<RULE>(w[2], w[3], sc, byte);
                    if (bad) { c0 = 0; c1 = 0; }
                    if (ract) *reinterpret_cast<uint2*>(codes_r + e0) = make_uint2(c0, c1);
                    if (STATS) err8(w, c0, c1, sc, unused, se_r, false);
                    if (STATS == 2) {
                        const unsigned bo = scale_byte<kFP4, RULE>(am);
                        const float sco = scale_operand(bo);
                        err4(w, enc4(w[0], w[1], w[2], w[3], sco), sco, unused, so_r, false);
                    }
                } else {
                    unsigned c4 = enc4(w[0], w[1], w[2], w[3], sc);
                    if (bad) c4 = 0;
                    if (ract) *reinterpret_cast<unsigned*>(codes_r + (e0 >> 1)) = c4;
                    if (STATS) err4(w, c4, sc, unused, se_r, false);
                    if (STATS == 2) {
                        const unsigned bo = scale_byte<kFP8, RULE>(am);
                        const float sco = scale_operand(bo);
                        err8(w, enc8<RULE>(w[0], w[1], sco, bo), enc8<RULE>(w[2], w[3], sco, bo), sco, unused, so_r, false);
                    }
                }
                // the four block bytes of this row's 128-column group: one dword of the grouped copy and,
                // when rows hold a whole number of groups, of the row-major array too
                const unsigned p1 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)byte, 0x104, 0xF, 0xF, true);   // lane + 4
                const unsigned p2 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)byte, 0x108, 0xF, 0xF, true);   // lane + 8
                const unsigned p3 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)byte, 0x10C, 0xF, 0xF, true);   // lane + 12
                const unsigned d = byte | (p1 << 8) | (p2 << 16) | (p3 << 24);
                if (ract && (lane & 15) == 0) {
                    if ((nblk & 3) == 0) *reinterpret_cast<unsigned*>(scales_r + (int64_t)row * nblk + cg * 4) = d;
                    if (g4_r) *reinterpret_cast<unsigned*>(g4_r + ((int64_t)cg * kpitch_r + row) * 4) = d;
                }
                if ((nblk & 3) != 0 && ract && (lane & 3) == 0)
                    scales_r[(int64_t)row * nblk + (rcol >> 5)] = (uint8_t)byte;
            }
        };
        if (PREFETCH) {
            unsigned cv0[32], cv1[32];
            uint4 rv0[8], rv1[8];
            if (k_first < nb) fetch(k_first, cv0, rv0);
            for (int k = k_first; k < nb; k += 2 * KSTEP) {
                if (k + KSTEP < nb) fetch(k + KSTEP, cv1, rv1);
                work(k, cv0, rv0);
                if (k + KSTEP < nb) {
                    if (k + 2 * KSTEP < nb) fetch(k + 2 * KSTEP, cv0, rv0);
                    work(k + KSTEP, cv1, rv1);
                }
            }
        } else {
            for (int k = k_first; k < nb; k += KSTEP) {
                unsigned cv[32];
                uint4 rv[8];
                fetch(k, cv, rv);
                work(k, cv, rv);
            }
        }
        if (COOP) {
            __syncthreads();                                   // all tiles of the unit are staged
            for (int g = wib; 4 * g < nb; g += kWavesPerBlock) {
                const int last = min(3, nb - 1 - 4 * g);
                unsigned lo = 0, hi = 0;
                for (int i = 0; i <= last; ++i) {
                    const unsigned v = *reinterpret_cast<const uint16_t*>(scale_stage + (4 * g + i) * kColsPerWave + 2 * lane);
                    lo |= (v & 0xFFu) << (8 * i);
                    hi |= (v >> 8) << (8 * i);
                }
                store_col_scales(rb0 + 4 * g, last, lo, hi);
            }
        }
#pragma unroll
        for (int it = k_first; it < kColsPerWave * CPR / 64; it += KSTEP) {
            const int idx = it * 64 + lane;
            const int row = idx / CPR, chunk = idx % CPR;
            const uint4 q = *reinterpret_cast<const uint4*>(reg + row * ROWB + ((chunk ^ ((row >> 1) & (CPR - 1))) * 16));
            const int cc = cg * kColsPerWave + row;
            const int blk = FMT_C == kFP8 ? chunk >> 1 : chunk;
            if (cc < cols && blk < nb)
                *reinterpret_cast<uint4*>(codes_c + (int64_t)cc * out_row_bytes + (int64_t)ru * ROWB + chunk * 16) = q;
        }
        if (COOP) __syncthreads();                             // the staging areas go to the next unit
    }
    if (STATS) {
        s0 = wave_sum(s0);
        se_r = wave_sum(se_r);
        se_c = wave_sum(se_c);
        if (STATS == 2) { so_r = wave_sum(so_r); so_c = wave_sum(so_c); }
        if (lane == 0) {
            float* p = partials + wave * 6;
            p[0] = s0; p[1] = FMT_R == kFP4 ? se_r : so_r; p[2] = FMT_R == kFP8 ? se_r : so_r;
            p[3] = s0; p[4] = FMT_C == kFP4 ? se_c : so_c; p[5] = FMT_C == kFP8 ? se_c : so_c;
        }
    }
}

// Statistics only, both formats, column blocks.  Grid: blockIdx.y = row split; a wave owns a
// column group and the rows of its split, so per-column sums stay in the lane.
template <int RULE>
__global__ __launch_bounds__(256) void stats_col_kernel(const uint16_t* __restrict__ x, int rows,
                                                        int cols, int64_t ld, int nsplit,
                                                        float* __restrict__ partials,
                                                        float* __restrict__ line_partials)
{
    const int lane = threadIdx.x & 63;
    const int wave_x = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    const int nwaves_x = gridDim.x * kWavesPerBlock;
    const int split = blockIdx.y;
    const int ncg = (cols + kColsPerWave - 1) / kColsPerWave;
    const int nrb = rows / kBlock;
    const int rb0 = (int)((int64_t)nrb * split / nsplit), rb1 = (int)((int64_t)nrb * (split + 1) / nsplit);
    float t0 = 0.f, t4 = 0.f, t8 = 0.f;
    for (int cg = wave_x; cg < ncg; cg += nwaves_x) {
        const int c = cg * kColsPerWave + lane * 2;
        const bool act = c < cols;
        float a0[2] = {0.f, 0.f}, a4[2] = {0.f, 0.f}, a8[2] = {0.f, 0.f};
        for (int rb = rb0; rb < rb1; ++rb) {
            ColBlock b;
            load_col_block(x + (int64_t)rb * kBlock * ld + c, ld, act, b);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const unsigned* w = h ? b.hi : b.lo;
                const unsigned am = h ? b.am_hi : b.am_lo;
                const unsigned b8 = scale_byte<kFP8, RULE>(am), b4 = scale_byte<kFP4, RULE>(am);
                const float sc8 = scale_operand(b8), sc4 = scale_operand(b4);
                float dummy = 0.f;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const unsigned c0 = enc8<RULE>(w[4 * k], w[4 * k + 1], sc8, b8);
                    const unsigned c1 = enc8<RULE>(w[4 * k + 2], w[4 * k + 3], sc8, b8);
                    err8(w + 4 * k, c0, c1, sc8, a0[h], a8[h], true);
                    const unsigned c4 = enc4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3], sc4);
                    err4(w + 4 * k, c4, sc4, dummy, a4[h], false);
                }
                if (b8 == 0xFFu) { a4[h] = __builtin_nanf(""); a8[h] = __builtin_nanf(""); }
            }
        }
        if (line_partials && act) {
            float* lp = line_partials + ((int64_t)split * cols + c) * 3;
            lp[0] = a0[0]; lp[1] = a4[0]; lp[2] = a8[0];
            lp[3] = a0[1]; lp[4] = a4[1]; lp[5] = a8[1];
        }
        t0 += a0[0] + a0[1]; t4 += a4[0] + a4[1]; t8 += a8[0] + a8[1];
    }
    t0 = wave_sum(t0); t4 = wave_sum(t4); t8 = wave_sum(t8);
    if (lane == 0) {
        float* p = partials + ((int64_t)split * nwaves_x + wave_x) * 3;
        p[0] = t0; p[1] = t4; p[2] = t8;
    }
}

// Statistics for BOTH block directions from one read of the matrix (the complete Step-1 record of a tensor:
// its forward operands are blocked along rows, its backward ones down columns, Sec. 2.2).
// Grid and ownership as in stats_col_kernel: a wave owns 128 columns and a range of 32-row blocks; a lane
// reads two adjacent columns of every row.  The column-direction errors come straight from those registers
// (a column's block never leaves the lane).  For the row direction the raw 32 x 128 tile goes through the
// wave's 8 KB of LDS and comes back as eight 16-byte pieces per lane: two whole 32-element row blocks, so that
// the row direction, too, forms a block's maximum and scales inside one lane.  LDS operations
// of one wave execute in order, so no barrier is needed between the writes and the reads.
// partials: [waves][6] = {sum x^2, row err4, row err8, sum x^2, col err4, col err8}.
template <int RULE>
__global__ __launch_bounds__(256) void stats_both_kernel(const uint16_t* __restrict__ x, int rows,
                                                         int cols, int64_t ld, int nsplit,
                                                         float* __restrict__ partials)
{
    __shared__ __attribute__((aligned(16))) unsigned tile[kWavesPerBlock][kBlock * 64];
    const int lane = threadIdx.x & 63;
    unsigned* const raw = tile[threadIdx.x >> 6];
    const int wave_x = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    const int nwaves_x = gridDim.x * kWavesPerBlock;
    const int split = blockIdx.y;
    const int ncg = (cols + kColsPerWave - 1) / kColsPerWave;
    const int nrb = rows / kBlock;
    const int rb0 = (int)((int64_t)nrb * split / nsplit), rb1 = (int)((int64_t)nrb * (split + 1) / nsplit);
    float t0 = 0.f, r4 = 0.f, r8 = 0.f, c4 = 0.f, c8 = 0.f;
    bool bad = false;
    // LDS image of the raw tile: row i holds its sixteen 16-byte pieces at positions piece ^ (i % 4), so that the
    // 16 lanes served together by a 16-byte read (4 rows x 4 blocks) fall into 16 different bank groups.
    int wpos[4], rpos[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        wpos[t] = (((lane >> 2) ^ t) << 2) | (lane & 3);                                   // dword lane of a row with i % 4 == t
        rpos[t] = (lane >> 2) * 64 + ((((lane & 3) * 4 + t) ^ ((lane >> 2) & 3)) << 2);    // piece t of block lane % 4, row lane / 4
    }
    for (int cg = wave_x; cg < ncg; cg += nwaves_x) {
        const int c = cg * kColsPerWave + lane * 2;
        const bool act = c < cols;
        for (int rb = rb0; rb < rb1; ++rb) {
            const uint16_t* p = x + (int64_t)rb * kBlock * ld + c;
            unsigned v[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) v[i] = act ? ld4(p + (int64_t)i * ld) : 0u;
#pragma unroll
            for (int i = 0; i < 32; ++i) raw[i * 64 + wpos[i & 3]] = v[i];
            // ---- column direction ----
            unsigned m = 0;
#pragma unroll
            for (int i = 0; i < 32; ++i) m = pk_max_u16(m, v[i] & 0x7FFF7FFFu);
            unsigned w[16];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int k = 0; k < 16; ++k)
                    w[k] = __builtin_amdgcn_perm(v[2 * k + 1], v[2 * k], h ? 0x07060302u : 0x05040100u);
                const unsigned am = h ? m >> 16 : m & 0xFFFFu;
                const unsigned b8 = scale_byte<kFP8, RULE>(am), b4 = scale_byte<kFP4, RULE>(am);
                const float sc8 = scale_operand(b8), sc4 = scale_operand(b4);
                float dummy = 0.f;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const unsigned e0 = enc8<RULE>(w[4 * k], w[4 * k + 1], sc8, b8);
                    const unsigned e1 = enc8<RULE>(w[4 * k + 2], w[4 * k + 3], sc8, b8);
                    err8(w + 4 * k, e0, e1, sc8, t0, c8, true);
                    const unsigned e4 = enc4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3], sc4);
                    err4(w + 4 * k, e4, sc4, dummy, c4, false);
                }
                bad |= b8 == 0xFFu;
            }
            // ---- row direction: the lane takes two whole blocks, block lane % 4 of tile rows lane / 4 and
            //      16 + lane / 4, as four 16-byte pieces each, so that a block's maximum and its two scales are
            //      formed once per 32 elements, inside the lane ----
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                uint4 q[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) q[k] = *reinterpret_cast<const uint4*>(raw + h * 16 * 64 + rpos[k]);
                unsigned m = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    m = pk_max_u16(m, pk_max_u16(pk_max_u16(q[k].x & 0x7FFF7FFFu, q[k].y & 0x7FFF7FFFu),
                                                 pk_max_u16(q[k].z & 0x7FFF7FFFu, q[k].w & 0x7FFF7FFFu)));
                const unsigned lo = m & 0xFFFFu, hi = m >> 16;
                const unsigned am = lo > hi ? lo : hi;
                const unsigned b8 = scale_byte<kFP8, RULE>(am), b4 = scale_byte<kFP4, RULE>(am);
                const float sc8 = scale_operand(b8), sc4 = scale_operand(b4);
                float dummy = 0.f;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const unsigned ww[4] = {q[k].x, q[k].y, q[k].z, q[k].w};
                    const unsigned e0 = enc8<RULE>(ww[0], ww[1], sc8, b8), e1 = enc8<RULE>(ww[2], ww[3], sc8, b8);
                    const unsigned e4 = enc4(ww[0], ww[1], ww[2], ww[3], sc4);
                    err8(ww, e0, e1, sc8, dummy, r8, false);
                    err4(ww, e4, sc4, dummy, r4, false);
                }
                bad |= b8 == 0xFFu;
            }
        }
    }
    if (bad) { r4 = c4 = r8 = c8 = __builtin_nanf(""); }     // a non-finite element poisons every error sum of the wave
    t0 = wave_sum(t0); r4 = wave_sum(r4); r8 = wave_sum(r8); c4 = wave_sum(c4); c8 = wave_sum(c8);
    if (lane == 0) {
        float* pp = partials + ((int64_t)split * nwaves_x + wave_x) * 6;
        pp[0] = t0; pp[1] = r4; pp[2] = r8; pp[3] = t0; pp[4] = c4; pp[5] = c8;
    }
}

// Second stage for stats_both_kernel: sums of n partials [n][6] in double, fixed order; out_row and out_col
// receive three doubles each.
__global__ __launch_bounds__(1024) void reduce_both_kernel(const float* __restrict__ partials, int n,
                                                           double* __restrict__ out_row, double* __restrict__ out_col,
                                                           int mode_row, int mode_col)
{
    __shared__ double sh[6][1024];
    double a[6] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    for (int i = threadIdx.x; i < n; i += 1024)
        for (int j = 0; j < 6; ++j) a[j] += (double)partials[(size_t)i * 6 + j];
    for (int j = 0; j < 6; ++j) sh[j][threadIdx.x] = a[j];
    __syncthreads();
    for (int st = 512; st > 0; st >>= 1) {
        if ((int)threadIdx.x < st)
            for (int j = 0; j < 6; ++j) sh[j][threadIdx.x] += sh[j][threadIdx.x + st];
        __syncthreads();
    }
    // mode 0: all three sums; mode 1 (fused FP4): the FP8 field is NaN; mode 2 (fused FP8): the FP4 field is NaN
    if (threadIdx.x < 6) {
        const int f = threadIdx.x % 3;
        const int mode = threadIdx.x < 3 ? mode_row : mode_col;
        double* out = threadIdx.x < 3 ? out_row : out_col;
        const bool absent = (mode == 1 && f == 2) || (mode == 2 && f == 1);
        if (out) out[f] = absent ? __builtin_nan("") : sh[threadIdx.x][0];
    }
}

// Second stage: sum n per-wave partials [n][3] in double, fixed order, one block of 1024 threads.
// Thread t owns partials 8t .. 8t+7 (and the same window every 8192 partials), read as six float4.
// mode 0: out = {p0, p1, p2}; mode 1 (fused FP4): out = {p0, p1, NaN}; mode 2 (fused FP8): {p0, NaN, p1}.
constexpr int kReduceThreads = 1024;
__global__ __launch_bounds__(kReduceThreads) void reduce_partials_kernel(const float* __restrict__ partials, int n,
                                                                         int mode, double* __restrict__ out)
{
    __shared__ double sh[3][kReduceThreads];
    double a[3] = {0.0, 0.0, 0.0};
    for (int base = threadIdx.x * 8; base < n; base += kReduceThreads * 8) {
        if (base + 8 <= n) {
            const float4* p = reinterpret_cast<const float4*>(partials + (size_t)base * 3);
            float v[24];
#pragma unroll
            for (int k = 0; k < 6; ++k) { const float4 q = p[k]; v[4 * k] = q.x; v[4 * k + 1] = q.y; v[4 * k + 2] = q.z; v[4 * k + 3] = q.w; }
#pragma unroll
            for (int k = 0; k < 24; ++k) a[k % 3] += (double)v[k];
        } else {
            for (int i = base; i < n; ++i)
                for (int j = 0; j < 3; ++j) a[j] += (double)partials[(size_t)i * 3 + j];
        }
    }
    for (int j = 0; j < 3; ++j) sh[j][threadIdx.x] = a[j];
    __syncthreads();
    for (int s = kReduceThreads / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s)
            for (int j = 0; j < 3; ++j) sh[j][threadIdx.x] += sh[j][threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double nan = __builtin_nan("");
        if (mode == 0)      { out[0] = sh[0][0]; out[1] = sh[1][0]; out[2] = sh[2][0]; }
        else if (mode == 1) { out[0] = sh[0][0]; out[1] = sh[1][0]; out[2] = nan; }
        else                { out[0] = sh[0][0]; out[1] = nan;      out[2] = sh[1][0]; }
    }
}

// Per-column sums: add the row splits in order.
__global__ __launch_bounds__(256) void reduce_lines_kernel(const float* __restrict__ line_partials, int nsplit,
                                                           int64_t n3, float* __restrict__ per_line)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n3) return;
    double a = 0.0;
    for (int s = 0; s < nsplit; ++s) a += (double)line_partials[(int64_t)s * n3 + i];
    per_line[i] = (float)a;
}

int col_splits(int64_t rows, int64_t cols, int* gx)
{
    const int ncg = (int)((cols + kColsPerWave - 1) / kColsPerWave);
    int g = (ncg + kWavesPerBlock - 1) / kWavesPerBlock;
    if (g > kStreamBlocks) g = kStreamBlocks;
    const int nrb = (int)(rows / kBlock);
    int64_t want = kStreamWaves / ((int64_t)g * kWavesPerBlock);
    if (want < 1) want = 1;
    if (want > kMaxColSplits) want = kMaxColSplits;
    if (want > nrb) want = nrb > 0 ? nrb : 1;
    *gx = g;
    return (int)want;
}

}  // namespace

size_t workspace_bytes(int64_t rows, int64_t cols)
{
    (void)rows;
    return stream_workspace_bytes(cols);
}

// Workgroups for `units` equal work units that waves take in turn: as many waves as give every wave the
// same number of units (the last one possibly fewer), at most kStreamWaves.  11008 units on 8192 waves would
// leave three quarters of the device idle during the second turn; 5504 waves take two units each.
static int balanced_blocks(int64_t units)
{
    if (units <= 0) return 1;
    const int64_t per_wave = (units + kStreamWaves - 1) / kStreamWaves;
    const int64_t waves = (units + per_wave - 1) / per_wave;
    return (int)((waves + kWavesPerBlock - 1) / kWavesPerBlock);
}

// Returns the number of workgroups launched (= partial-sum slots used, times kWavesPerBlock).
template <int FMT, int RULE, bool STATS, bool SR = false>
static int launch_q(const QuantArgs& a, float* partials, hipStream_t s)
{
    const uint2 seed = make_uint2((unsigned)a.sr_seed, (unsigned)(a.sr_seed >> 32));
    int blocks;
    // pitch of the block-major scale copy = padded number of STORED rows
    if (a.axis == 0) {
        blocks = balanced_blocks(((a.rows + kUnroll - 1) / kUnroll) * ((a.cols + kSeg - 1) / kSeg));
        hipLaunchKernelGGL((quant_row_kernel<FMT, RULE, STATS, SR>), dim3(blocks), dim3(256), 0, s,
                           a.x, (int)a.rows, (int)a.cols, a.ld, a.codes, a.scales, a.scales_g4,
                           g4_pitch(a.rows), partials, seed);
    } else {
        const int64_t nrb = a.rows / kBlock;
        const int rbu = (FMT == kFP8 || SR) ? kRowBlocksPerUnit : 2 * kRowBlocksPerUnit;       // as in quant_col_kernel
        const int64_t units = ((a.cols + kColsPerWave - 1) / kColsPerWave) * ((nrb + rbu - 1) / rbu);
        // a workgroup per unit (see quant_col_kernel); SNIP_QUANT_COL_UNIT=wave|workgroup, read at every call, fixes
        // the choice for tests and measurements
        bool coop = true;
        if (const char* e = getenv("SNIP_QUANT_COL_UNIT")) coop = !(e[0] == 'w' && e[1] == 'a');
        if (coop) {
            blocks = (int)(units < kStreamBlocks ? units : kStreamBlocks);
            hipLaunchKernelGGL((quant_col_kernel<FMT, RULE, STATS, SR, true>), dim3(blocks), dim3(256), 0, s,
                               a.x, (int)a.rows, (int)a.cols, a.ld, a.codes, a.scales, a.scales_g4,
                               g4_pitch(a.cols), partials, seed);
        } else {
            blocks = balanced_blocks(units);
            hipLaunchKernelGGL((quant_col_kernel<FMT, RULE, STATS, SR, false>), dim3(blocks), dim3(256), 0, s,
                               a.x, (int)a.rows, (int)a.cols, a.ld, a.codes, a.scales, a.scales_g4,
                               g4_pitch(a.cols), partials, seed);
        }
    }
    return blocks;
}

hipError_t launch_quantize(const QuantArgs& a, hipStream_t s)
{
    if (a.rows == 0 || a.cols == 0) {
        if (a.stats) {
            hipLaunchKernelGGL(reduce_partials_kernel, dim3(1), dim3(kReduceThreads), 0, s,
                               (const float*)a.workspace, 0, a.fmt == kFP4 ? 1 : 2, a.stats);
        }
        return hipGetLastError();
    }
    float* partials = (float*)a.workspace;
    const bool st = a.stats != nullptr;
    if (a.stochastic) {
        if (a.fmt != kFP4 || st) return hipErrorInvalidValue;
        if (a.rule == 0) launch_q<kFP4, 0, false, true>(a, partials, s);
        else             launch_q<kFP4, 1, false, true>(a, partials, s);
        return hipGetLastError();
    }
    const int key = (a.fmt << 2) | (a.rule << 1) | (st ? 1 : 0);
    int blocks = 0;
    switch (key) {
        case 0: blocks = launch_q<kFP8, 0, false>(a, partials, s); break;
        case 1: blocks = launch_q<kFP8, 0, true>(a, partials, s); break;
        case 2: blocks = launch_q<kFP8, 1, false>(a, partials, s); break;
        case 3: blocks = launch_q<kFP8, 1, true>(a, partials, s); break;
        case 4: blocks = launch_q<kFP4, 0, false>(a, partials, s); break;
        case 5: blocks = launch_q<kFP4, 0, true>(a, partials, s); break;
        case 6: blocks = launch_q<kFP4, 1, false>(a, partials, s); break;
        case 7: blocks = launch_q<kFP4, 1, true>(a, partials, s); break;
        default: return hipErrorInvalidValue;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (st) {
        hipLaunchKernelGGL(reduce_partials_kernel, dim3(1), dim3(kReduceThreads), 0, s,
                           (const float*)partials, blocks * kWavesPerBlock, a.fmt == kFP4 ? 1 : 2, a.stats);
        e = hipGetLastError();
    }
    return e;
}

// With the statistics of both formats: up to this many units of four tiles (half as many again of eight) a tensor is
// quantized with one workgroup per unit (COOP), see launch_quantize_both.
constexpr int kCoopMaxUnits = 1024;

template <int FMT_R, int FMT_C, int RULE, int STATS>
static void launch_qb(const QuantBothArgs& a, float* partials, int blocks, bool coop, hipStream_t s)
{
    if (coop)
        hipLaunchKernelGGL((quant_both_kernel<FMT_R, FMT_C, RULE, STATS, true>), dim3(blocks), dim3(256), 0, s,
                           a.x, (int)a.rows, (int)a.cols, a.ld, a.codes_r, a.scales_r, a.g4_r, g4_pitch(a.rows),
                           a.codes_c, a.scales_c, a.g4_c, g4_pitch(a.cols), partials);
    else
        hipLaunchKernelGGL((quant_both_kernel<FMT_R, FMT_C, RULE, STATS, false>), dim3(blocks), dim3(256), 0, s,
                           a.x, (int)a.rows, (int)a.cols, a.ld, a.codes_r, a.scales_r, a.g4_r, g4_pitch(a.rows),
                           a.codes_c, a.scales_c, a.g4_c, g4_pitch(a.cols), partials);
}

hipError_t launch_quantize_both(const QuantBothArgs& a, hipStream_t s)
{
    float* partials = (float*)a.workspace;
    const bool st = a.stats_r != nullptr;
    // second stage: which field of each triple is "not computed" (NaN); none when both formats are wanted
    const int mode_r = a.both_formats ? 0 : (a.fmt_r == kFP4 ? 1 : 2), mode_c = a.both_formats ? 0 : (a.fmt_c == kFP4 ? 1 : 2);
    if (a.rows == 0 || a.cols == 0) {
        if (st) hipLaunchKernelGGL(reduce_both_kernel, dim3(1), dim3(1024), 0, s, (const float*)partials, 0, a.stats_r, a.stats_c, mode_r, mode_c);
        return hipGetLastError();
    }
    const int64_t nrb = a.rows / kBlock;
    const int rbu = a.fmt_c == kFP8 ? kRowBlocksPerUnit : 2 * kRowBlocksPerUnit;           // as in quant_both_kernel
    const int64_t units = ((a.cols + kColsPerWave - 1) / kColsPerWave) * ((nrb + rbu - 1) / rbu);
    // Work distribution.  One workgroup per unit (its four waves share the unit's tiles, 17 KB of LDS per workgroup,
    // so more waves are resident) is the faster form except with the statistics of both formats, which fill the
    // registers: there it pays only while a wave per unit would leave SIMDs without work (measured break-even: 1024
    // units of four tiles, 1536 of eight).  SNIP_QUANT_BOTH_UNIT=wave|workgroup in the environment, read at every
    // call, fixes the choice for tests and measurements.
    const int mode = !st ? 0 : (a.both_formats ? 2 : 1);
    bool coop = mode != 2 || units <= (a.fmt_c == kFP8 ? kCoopMaxUnits : kCoopMaxUnits + kCoopMaxUnits / 2);
    if (const char* e = getenv("SNIP_QUANT_BOTH_UNIT")) {
        if (e[0] == 'w' && e[1] == 'a') coop = false;
        if (e[0] == 'w' && e[1] == 'o') coop = true;
    }
    // (a workgroup walks units blockIdx.x, blockIdx.x + gridDim.x, ...; the grid stays within the partial-sum slots)
    const int blocks = coop ? (int)(units < kStreamBlocks ? units : kStreamBlocks) : balanced_blocks(units);
    const int key = (a.fmt_r << 4) | (a.fmt_c << 3) | (a.rule << 2) | mode;
    switch (key) {
#define SNIP_QB_CASE(FR, FC, RU) \
        case ((FR) << 4) | ((FC) << 3) | ((RU) << 2) | 0: launch_qb<FR, FC, RU, 0>(a, partials, blocks, coop, s); break; \
        case ((FR) << 4) | ((FC) << 3) | ((RU) << 2) | 1: launch_qb<FR, FC, RU, 1>(a, partials, blocks, coop, s); break; \
        case ((FR) << 4) | ((FC) << 3) | ((RU) << 2) | 2: launch_qb<FR, FC, RU, 2>(a, partials, blocks, coop, s); break;
        SNIP_QB_CASE(0, 0, 0) SNIP_QB_CASE(0, 0, 1) SNIP_QB_CASE(0, 1, 0) SNIP_QB_CASE(0, 1, 1)
        SNIP_QB_CASE(1, 0, 0) SNIP_QB_CASE(1, 0, 1) SNIP_QB_CASE(1, 1, 0) SNIP_QB_CASE(1, 1, 1)
#undef SNIP_QB_CASE
        default: return hipErrorInvalidValue;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (st) {
        hipLaunchKernelGGL(reduce_both_kernel, dim3(1), dim3(1024), 0, s, (const float*)partials, blocks * kWavesPerBlock,
                           a.stats_r, a.stats_c, mode_r, mode_c);
        e = hipGetLastError();
    }
    return e;
}

hipError_t launch_stats_both(const StatsArgs& a, double* out_col, hipStream_t s)
{
    float* partials = (float*)a.workspace;
    if (a.rows == 0 || a.cols == 0) {
        hipLaunchKernelGGL(reduce_both_kernel, dim3(1), dim3(1024), 0, s, (const float*)partials, 0, a.stats, out_col, 0, 0);
        return hipGetLastError();
    }
    int gx;
    const int nsplit = col_splits(a.rows, a.cols, &gx);
    if (a.rule == 0)
        hipLaunchKernelGGL((stats_both_kernel<0>), dim3(gx, nsplit), dim3(256), 0, s, a.x, (int)a.rows, (int)a.cols, a.ld, nsplit, partials);
    else
        hipLaunchKernelGGL((stats_both_kernel<1>), dim3(gx, nsplit), dim3(256), 0, s, a.x, (int)a.rows, (int)a.cols, a.ld, nsplit, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(reduce_both_kernel, dim3(1), dim3(1024), 0, s, (const float*)partials, gx * kWavesPerBlock * nsplit,
                       a.stats, out_col, 0, 0);
    return hipGetLastError();
}

hipError_t launch_stats(const StatsArgs& a, hipStream_t s)
{
    float* partials = (float*)a.workspace;
    if (a.rows == 0 || a.cols == 0) {
        hipLaunchKernelGGL(reduce_partials_kernel, dim3(1), dim3(kReduceThreads), 0, s, (const float*)partials, 0, 0, a.stats);
        return hipGetLastError();
    }
    int npart;
    if (a.axis == 0) {
        const int blocks = balanced_blocks(a.rows);             // a wave per row
        if (a.rule == 0)
            hipLaunchKernelGGL((stats_row_kernel<0>), dim3(blocks), dim3(256), 0, s,
                               a.x, (int)a.rows, (int)a.cols, a.ld, partials, a.per_line);
        else
            hipLaunchKernelGGL((stats_row_kernel<1>), dim3(blocks), dim3(256), 0, s,
                               a.x, (int)a.rows, (int)a.cols, a.ld, partials, a.per_line);
        npart = blocks * kWavesPerBlock;
    } else {
        int gx;
        const int nsplit = col_splits(a.rows, a.cols, &gx);
        float* lines = a.per_line ? (float*)((char*)a.workspace + kPartialBytes) : nullptr;
        if (a.rule == 0)
            hipLaunchKernelGGL((stats_col_kernel<0>), dim3(gx, nsplit), dim3(256), 0, s,
                               a.x, (int)a.rows, (int)a.cols, a.ld, nsplit, partials, lines);
        else
            hipLaunchKernelGGL((stats_col_kernel<1>), dim3(gx, nsplit), dim3(256), 0, s,
                               a.x, (int)a.rows, (int)a.cols, a.ld, nsplit, partials, lines);
        npart = gx * kWavesPerBlock * nsplit;
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (a.per_line) {
            const int64_t n3 = a.cols * 3;
            hipLaunchKernelGGL(reduce_lines_kernel, dim3((unsigned)((n3 + 255) / 256)), dim3(256), 0, s,
                               (const float*)lines, nsplit, n3, a.per_line);
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3(1), dim3(kReduceThreads), 0, s, (const float*)partials, npart, 0, a.stats);
    return hipGetLastError();
}

}  // namespace snip
