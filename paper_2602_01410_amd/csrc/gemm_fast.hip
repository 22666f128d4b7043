// Large-tile variant of the block-scaled GEMM for contraction extents that are multiples of 128.
//
//   workgroup tile 256 x 256, 8 waves (2 x 4), wave tile 128 (A rows) x 64 (B rows)
//   pipeline stage = 128 contraction elements; operand tiles and their scale dwords are copied
//   global -> LDS by the load unit itself (global_load_lds), never through VGPRs; a ring of
//   2-4 stage buffers keeps up to 3 stages in flight; one barrier per stage
//   LDS rows are unpadded; the 16-byte chunks of a row are XOR-swizzled (on the global-address
//   side of the copy) so that the 16 lanes served together by a ds_read_b128 hit 16 different
//   bank groups
//
// See gemm.hip for the register layout of v_mfma_scale_f32_32x32x64_f8f6f4.
#include "snip_internal.h"

namespace snip {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

constexpr int TM = 256, TN = 256;       // workgroup tile
constexpr int NWAVE = 8, NT = NWAVE * 64;
constexpr int WTM = 128, WTN = 64;      // wave tile
constexpr int MB = WTM / 32, NB = WTN / 32;

#define SNIP_GLDS16(gp, lp) __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gp), (__attribute__((address_space(3))) void*)(lp), 16, 0, 0)
#define SNIP_GLDS4(gp, lp) __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gp), (__attribute__((address_space(3))) void*)(lp), 4, 0, 0)
// s_waitcnt vmcnt(n), other counters untouched (gfx9 encoding: vmcnt[3:0], expcnt[6:4], lgkmcnt[11:8], vmcnt[5:4] in [15:14])
#define SNIP_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | ((((n) >> 4) & 3) << 14))

template <int FA, int FB> struct FCfg {
    static constexpr int KE = 128;                               // contraction elements per stage
    static constexpr int SBA = FA == kFP8 ? 128 : 64;            // code bytes per row per stage
    static constexpr int SBB = FB == kFP8 ? 128 : 64;
    static constexpr int NST = (SBA + SBB == 128) ? 4 : (SBA + SBB == 192 ? 3 : 2);
    static constexpr int LA = TM * SBA / 1024 / NWAVE;           // 16-byte copy instructions per wave per stage
    static constexpr int LB = TN * SBB / 1024 / NWAVE;
    static constexpr int L = LA + LB + 1;                        // + one scale dword
    static constexpr int A_BYTES = TM * SBA, B_BYTES = TN * SBB;
};

// Swizzle: chunk position p of `row` holds logical chunk p ^ f(row); f makes the 16/CPR rows that share
// a 256-byte bank span use different positions.
template <int SB> __device__ __forceinline__ int swz(int row)
{
    constexpr int CPR = SB / 16;
    return (row / (16 / CPR)) % CPR;
}

template <int F, int SB>
__device__ __forceinline__ v8i read_frag(const uint8_t* tile, int rowblock_off, const int* off, int ks)
{
    v8i f = {0, 0, 0, 0, 0, 0, 0, 0};
    if (F == kFP8) {
        const uint4 a = *reinterpret_cast<const uint4*>(tile + rowblock_off + off[ks * 2 + 0]);
        const uint4 b = *reinterpret_cast<const uint4*>(tile + rowblock_off + off[ks * 2 + 1]);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    } else {
        const uint4 a = *reinterpret_cast<const uint4*>(tile + rowblock_off + off[ks]);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
    }
    return f;
}

template <int FA, int FB, bool OUT_F32>
__global__ __launch_bounds__(NT) void gemm_fast_kernel(const uint8_t* __restrict__ a_codes,
                                                       const uint8_t* __restrict__ a_scales,
                                                       const uint8_t* __restrict__ b_codes,
                                                       const uint8_t* __restrict__ b_scales,
                                                       int I, int J, int R, void* __restrict__ c_out, int64_t ldc,
                                                       int tiles_i, int tiles_j)
{
    using C = FCfg<FA, FB>;
    constexpr int NST = C::NST;
    // one object per ring slot, so that the compiler can tell a slot being filled from the slot being read
    __shared__ __attribute__((aligned(1024))) uint8_t sa0[C::A_BYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t sa1[C::A_BYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t sa2[NST > 2 ? C::A_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) uint8_t sa3[NST > 3 ? C::A_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) uint8_t sb0[C::B_BYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t sb1[C::B_BYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t sb2[NST > 2 ? C::B_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) uint8_t sb3[NST > 3 ? C::B_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) uint8_t ss0[2048];
    __shared__ __attribute__((aligned(1024))) uint8_t ss1[2048];
    __shared__ __attribute__((aligned(1024))) uint8_t ss2[NST > 2 ? 2048 : 16];
    __shared__ __attribute__((aligned(1024))) uint8_t ss3[NST > 3 ? 2048 : 16];
    uint8_t* const pa[4] = {sa0, sa1, sa2, sa3};
    uint8_t* const pb[4] = {sb0, sb1, sb2, sb3};
    uint8_t* const ps[4] = {ss0, ss1, ss2, ss3};

    // tile order: XCD-contiguous runs, then bands of 4 tile rows walked column by column
    const int nblk = tiles_i * tiles_j;
    int bid = blockIdx.x;
    {
        const int per = nblk / 8;
        if (bid < per * 8) bid = (bid % 8) * per + bid / 8;
    }
    const int band = 4;
    const int band_sz = band * tiles_j;
    const int b0 = bid / band_sz;
    const int rem = bid - b0 * band_sz;
    const int rows_in_band = min(band, tiles_i - b0 * band);
    const int ti = b0 * band + rem % rows_in_band;
    const int tj = rem / rows_in_band;
    const int i0 = ti * TM, j0 = tj * TN;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int r32 = lane & 31, g = lane >> 5;

    const int64_t a_row_bytes = FA == kFP8 ? R : R / 2;
    const int64_t b_row_bytes = FB == kFP8 ? R : R / 2;
    const int nkb = R / kBlock;
    const int nstage = R / C::KE;

    // ---- per-lane source addresses of the global->LDS copies (stage 0) ----
    const uint8_t* ga[C::LA];
    const uint8_t* gb[C::LB];
#pragma unroll
    for (int j = 0; j < C::LA; ++j) {
        constexpr int CPR = C::SBA / 16, RPI = 1024 / C::SBA;
        const int row = (wave * C::LA + j) * RPI + lane / CPR;
        const int c = (lane % CPR) ^ swz<C::SBA>(row);
        const int grow = min(i0 + row, I - 1);
        ga[j] = a_codes + (int64_t)grow * a_row_bytes + c * 16;
    }
#pragma unroll
    for (int j = 0; j < C::LB; ++j) {
        constexpr int CPR = C::SBB / 16, RPI = 1024 / C::SBB;
        const int row = (wave * C::LB + j) * RPI + lane / CPR;
        const int c = (lane % CPR) ^ swz<C::SBB>(row);
        const int grow = min(j0 + row, J - 1);
        gb[j] = b_codes + (int64_t)grow * b_row_bytes + c * 16;
    }
    const uint8_t* gs;
    {
        const int t = threadIdx.x;
        gs = t < TM ? a_scales + (int64_t)min(i0 + t, I - 1) * nkb : b_scales + (int64_t)min(j0 + t - TM, J - 1) * nkb;
    }

    auto issue = [&](int stage, int slot) {
        const int st = min(stage, nstage - 1);      // past the end: refill with the last stage (keeps the count of
                                                    // outstanding copies uniform; the data is never read)
#pragma unroll
        for (int j = 0; j < C::LA; ++j) SNIP_GLDS16(ga[j] + (int64_t)st * C::SBA, pa[slot] + (wave * C::LA + j) * 1024);
#pragma unroll
        for (int j = 0; j < C::LB; ++j) SNIP_GLDS16(gb[j] + (int64_t)st * C::SBB, pb[slot] + (wave * C::LB + j) * 1024);
        SNIP_GLDS4(gs + st * 4, ps[slot] + wave * 256);
    };

    // ---- per-lane LDS read offsets ----
    constexpr int NCA = FA == kFP8 ? 4 : 2, NCB = FB == kFP8 ? 4 : 2;   // chunk reads per stage per row block
    int offa[NCA], offb[NCB];
    {
        const int fa = swz<C::SBA>(r32), fb = swz<C::SBB>(r32);        // row-block bases are multiples of 32: f depends on r32 only
#pragma unroll
        for (int k = 0; k < NCA; ++k) {
            const int c = FA == kFP8 ? ((k >> 1) * 4 + (k & 1) * 2 + g) : (k * 2 + g);
            offa[k] = r32 * C::SBA + ((c ^ fa) * 16);
        }
#pragma unroll
        for (int k = 0; k < NCB; ++k) {
            const int c = FB == kFP8 ? ((k >> 1) * 4 + (k & 1) * 2 + g) : (k * 2 + g);
            offb[k] = r32 * C::SBB + ((c ^ fb) * 16);
        }
    }
    const int sca_off = (wm * WTM + r32) * 4, scb_off = (TM + wn * WTN + r32) * 4;

    v16f acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[a][b][k] = 0.f;

    auto compute = [&](int slot) {
        const uint8_t* ta = pa[slot] + wm * WTM * C::SBA;
        const uint8_t* tb = pb[slot] + wn * WTN * C::SBB;
        unsigned sa[MB], sb[NB];
#pragma unroll
        for (int m = 0; m < MB; ++m) sa[m] = *reinterpret_cast<const unsigned*>(ps[slot] + sca_off + m * 128) >> (8 * g);
#pragma unroll
        for (int n = 0; n < NB; ++n) sb[n] = *reinterpret_cast<const unsigned*>(ps[slot] + scb_off + n * 128) >> (8 * g);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v8i fa[MB], fb[NB];
#pragma unroll
            for (int m = 0; m < MB; ++m) fa[m] = read_frag<FA, C::SBA>(ta, m * 32 * C::SBA, offa, ks);
#pragma unroll
            for (int n = 0; n < NB; ++n) fb[n] = read_frag<FB, C::SBB>(tb, n * 32 * C::SBB, offb, ks);
            constexpr int ca = FB == kFP8 ? 0 : 4, cb = FA == kFP8 ? 0 : 4;
#pragma unroll
            for (int m = 0; m < MB; ++m)
#pragma unroll
                for (int n = 0; n < NB; ++n) {
                    if (ks == 0)
                        acc[m][n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[n], fa[m], acc[m][n], ca, cb, 0, (int)sb[n], 0, (int)sa[m]);
                    else
                        acc[m][n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[n], fa[m], acc[m][n], ca, cb, 2, (int)sb[n], 2, (int)sa[m]);
                }
        }
    };

    // ---- pipeline ----
#pragma unroll
    for (int st = 0; st < NST - 1; ++st) issue(st, st);
    for (int s0 = 0; s0 < nstage; s0 += NST) {
#pragma unroll
        for (int u = 0; u < NST; ++u) {
            const int s = s0 + u;
            if (s < nstage) {
                SNIP_WAIT_VM((NST - 2) * C::L);
                __builtin_amdgcn_s_barrier();
                issue(s + NST - 1, (u + NST - 1) % NST);
                compute(u);
            }
        }
    }
    SNIP_WAIT_VM(0);            // no copy may still be in flight when the LDS is handed to another workgroup
    __builtin_amdgcn_s_barrier();

    // ---- epilogue: lane owns row i; register quad q owns columns 8q + 4g .. +3 of each 32-wide block ----
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const int i = i0 + wm * WTM + m * 32 + r32;
        if (i >= I) continue;
#pragma unroll
        for (int n = 0; n < NB; ++n)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = j0 + wn * WTN + n * 32 + 8 * q + 4 * g;
                const float v0 = acc[m][n][4 * q + 0], v1 = acc[m][n][4 * q + 1];
                const float v2 = acc[m][n][4 * q + 2], v3 = acc[m][n][4 * q + 3];
                if (OUT_F32) {
                    float* p = reinterpret_cast<float*>(c_out) + (int64_t)i * ldc + j;
                    if (j + 3 < J) *reinterpret_cast<float4*>(p) = make_float4(v0, v1, v2, v3);
                    else { if (j < J) p[0] = v0; if (j + 1 < J) p[1] = v1; if (j + 2 < J) p[2] = v2; }
                } else {
                    __bf16* p = reinterpret_cast<__bf16*>(c_out) + (int64_t)i * ldc + j;
                    if (j + 3 < J) {
                        const float2_t lo = {v0, v1}, hi = {v2, v3};
                        const bf16x2 blo = __builtin_convertvector(lo, bf16x2), bhi = __builtin_convertvector(hi, bf16x2);
                        *reinterpret_cast<uint2*>(p) = make_uint2(__builtin_bit_cast(unsigned, blo), __builtin_bit_cast(unsigned, bhi));
                    } else {
                        if (j < J) p[0] = (__bf16)v0;
                        if (j + 1 < J) p[1] = (__bf16)v1;
                        if (j + 2 < J) p[2] = (__bf16)v2;
                    }
                }
            }
    }
}

template <int FA, int FB>
hipError_t launch_fast_t(const GemmArgs& a, hipStream_t s)
{
    const int ti = (int)((a.I + TM - 1) / TM), tj = (int)((a.J + TN - 1) / TN);
    const dim3 grid((unsigned)(ti * tj)), block(NT);
    if (a.out_fp32)
        hipLaunchKernelGGL((gemm_fast_kernel<FA, FB, true>), grid, block, 0, s, a.a_codes, a.a_scales, a.b_codes, a.b_scales,
                           (int)a.I, (int)a.J, (int)a.R, a.c, a.ldc, ti, tj);
    else
        hipLaunchKernelGGL((gemm_fast_kernel<FA, FB, false>), grid, block, 0, s, a.a_codes, a.a_scales, a.b_codes, a.b_scales,
                           (int)a.I, (int)a.J, (int)a.R, a.c, a.ldc, ti, tj);
    return hipGetLastError();
}

}  // namespace

bool gemm_fast_eligible(const GemmArgs& a)
{
    return a.R % 128 == 0 && a.R >= 128 && a.I > 128 && a.J > 128;
}

hipError_t launch_gemm_fast(const GemmArgs& a, hipStream_t s)
{
    if (a.fmt_a == kFP8 && a.fmt_b == kFP8) return launch_fast_t<kFP8, kFP8>(a, s);
    if (a.fmt_a == kFP8 && a.fmt_b == kFP4) return launch_fast_t<kFP8, kFP4>(a, s);
    if (a.fmt_a == kFP4 && a.fmt_b == kFP8) return launch_fast_t<kFP4, kFP8>(a, s);
    return launch_fast_t<kFP4, kFP4>(a, s);
}

}  // namespace snip
