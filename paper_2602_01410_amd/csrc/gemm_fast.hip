// Large-tile variant of the block-scaled GEMM, used when both operands carry the grouped scale copy
// (scales_g4) and the contraction extent is a multiple of the stage length.
//
//   workgroup tile 256 x 256, 8 waves (2 x 4), wave tile 128 (A rows) x 64 (B rows), fp32
//   accumulators in registers (128 per lane); for outputs that would leave compute units without a
//   tile, 256 x 128 with 4 x 2 waves of 64 x 64 (same code, other template argument).
//   A pipeline stage is 128 code bytes of every tile row for an FP8 operand and for FP4 x FP4
//   (256 contraction elements there), so every 128-byte line that is fetched is used whole.
//   Codes and scale dwords go global -> LDS through the load unit (global_load_lds), never through
//   VGPRs; two stage buffers.
//   The eight waves run a ping-pong schedule: the two waves of a SIMD alternate between reading
//   their operands of a phase from LDS and issuing that phase's MFMAs, one phase apart, separated by
//   workgroup barriers, so that the matrix core of every SIMD always has a wave with operands ready.
//   A wave issues its global -> LDS copies between the MFMAs of one of its MFMA phases, where issue
//   slots are free (an MFMA occupies the matrix core for 32 or 64 cycles, a copy instruction costs the
//   wave about 40); issued in front of the LDS reads they made that phase the longest of the four.
//   LDS rows are unpadded; the 16-byte chunks of a row are XOR-swizzled on the global-address side
//   of the copy so that the 16 lanes served together by a ds_read_b128 hit 16 different bank groups.
//   The result tile leaves through LDS as well: each wave transposes its 128 x 64 block so that the
//   global stores are 16 bytes per lane and 128 contiguous bytes per row.
//   The kernel is persistent: one workgroup per compute unit walks its tiles (dispatch ids blockIdx.x,
//   blockIdx.x + gridDim.x, ...) and treats their pipeline stages as one sequence, so the first stage of the
//   next tile is copied into the free stage buffer during the last stage of the current one and a tile's
//   start-up latency is paid once per workgroup, not once per tile.  The result tile is staged in the other
//   stage buffer (the one the last stage was read from), 64 KB at a time.
//
// What bounds it (hardware counters and variants of this kernel with one part removed, 16384 x 4096 x 4096 and
// 4096 x 4096 x 16384 on Gaussian data): the matrix cores are busy for 0.62-0.64 of the compute units' busy cycles
// and the shader clock (GRBM_GUI_ACTIVE over the launch duration) is 1.83 GHz (FP4) to 1.95 GHz (FP8) instead of 2.4;
// a loop of nothing but MFMAs on random operands runs at 1.64 / 2.03 GHz.  LDS is active a third of the time with
// 2 % bank-conflict cycles.  Leaving out the workgroup barriers changes nothing.  Leaving out the global -> LDS
// copies gains 20 % on random codes but 7 % on all-zero codes, half of the copies 8.5 %, and copies that always
// hit one L2-resident stage 5 %: what the copies cost is mostly clock (the chip slows down as more random bytes
// move through a compute unit), not latency and not misses.  The result stores cost 10 % at contraction extent
// 4096: all workgroups finish a tile together, 32 MB per round, and the next tile's copies queue behind them in
// the wave's memory counter.
//
// See gemm.hip for the register layout of v_mfma_scale_f32_32x32x64_f8f6f4.
#include "snip_internal.h"
#include <type_traits>
#include <cstdlib>

namespace snip {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int NWAVE = 8, NT = NWAVE * 64;
constexpr int TNP = 256;                // rows of the B tile's scale area (a 128-row B tile leaves half of it unused)

// Workgroup tile TM (A rows) x TN (B rows), split over the eight waves as (TM / WTM) x (TN / WTN) wave tiles.
template <int TM_, int TN_, int WTM_, int WTN_> struct TileCfg {
    static constexpr int TM = TM_, TN = TN_, WTM = WTM_, WTN = WTN_;
    static constexpr int WGN = TN / WTN;                   // waves along the B rows
    static constexpr int MB = WTM / 32, NB = WTN / 32;     // 32 x 32 MFMA blocks of a wave tile
    static_assert(TM == 256 && (TN == 256 || TN == 128), "copy shares and scale areas are laid out for these tiles");
    static_assert((TM / WTM) * (TN / WTN) == NWAVE, "eight waves");
};
// 256 x 256, 2 x 4 waves of 128 x 64: the largest tile the register file allows (fewest operand bytes per FLOP).
using TileBig = TileCfg<256, 256, 128, 64>;
// 256 x 128, 4 x 2 waves of 64 x 64: twice as many tiles for outputs that would leave compute units without one.
using TileWide = TileCfg<256, 128, 64, 64>;

// Global -> LDS copy issued by the load unit: lane i's 16 (or 4) bytes land at lds + 16*i (4*i); `lds` is
// wave-uniform and travels in M0.  Written as inline assembly on purpose: the compiler then keeps no
// scoreboard entry for these copies and never adds its own (conservative, count-zero) wait in front of LDS
// reads; completion is enforced by the explicit SNIP_WAIT_VM + barrier of the pipeline below.  The "memory"
// clobber tells the compiler that LDS contents change here.
__device__ __forceinline__ unsigned lds_addr(const void* p)
{
    return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}
// The source address is a wave-uniform 64-bit base (SGPR pair) plus a 32-bit per-lane byte offset.
__device__ __forceinline__ void glds16(const uint8_t* base, unsigned lane_off, unsigned lds)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_off), "s"(base), "s"(lds) : "memory", "m0");
}
__device__ __forceinline__ void glds4(const uint8_t* base, unsigned lane_off, unsigned lds)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" : : "v"(lane_off), "s"(base), "s"(lds) : "memory", "m0");
}
// s_waitcnt vmcnt(n), other counters untouched (gfx9 encoding: vmcnt[3:0], expcnt[6:4], lgkmcnt[11:8], vmcnt[5:4] in [15:14])
#define SNIP_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | ((((n) >> 4) & 3) << 14))

template <int FA, int FB, class T> struct FCfg {
    static constexpr int TM = T::TM, TN = T::TN;
    static constexpr bool BOTH4 = FA == kFP4 && FB == kFP4;
    static constexpr int KE = BOTH4 ? 256 : 128;                 // contraction elements per stage
    static constexpr int SBA = FA == kFP8 ? KE : KE / 2;         // code bytes per row per stage (128, or 64 for FP4 next to FP8)
    static constexpr int SBB = FB == kFP8 ? KE : KE / 2;
    static constexpr int KS = KE / 64;                           // MFMA steps per stage
    static constexpr int NG = KE / 128;                          // scale dwords (groups of 4 blocks) per row per stage
    static constexpr int NST = 2;                                // stage buffers
    static constexpr int A_BYTES = TM * SBA, B_BYTES = TN * SBB;
    static constexpr int S_BYTES = (TM + TNP) * NG * 4;          // scale dwords of one stage
    static constexpr int SLOT = A_BYTES + B_BYTES + S_BYTES;
    // Stage buffer 0 sits at the start of the LDS array and stage buffer 1 at its end; the result staging area is
    // the first or the last EPI_BYTES of the array, i.e. it covers the buffer of the tile's last stage (plus the
    // unused middle) and never reaches into the other buffer, which already receives the next tile.
    static constexpr int LDS_BYTES = 159 * 1024;
    static constexpr int SLOT1 = LDS_BYTES - SLOT;
    static constexpr int EPI_BYTES = 64 * 1024;
    static constexpr int LA = A_BYTES / 1024 / NWAVE;            // 16-byte copy instructions per wave per stage
    static constexpr int LB = B_BYTES / 1024 / NWAVE;
    static constexpr int LS = S_BYTES / 256 / NWAVE;             // 4-byte copy instructions per wave per stage
    static constexpr int L = LA + LB + LS;
    static_assert(SLOT1 % 1024 == 0 && SLOT <= SLOT1, "stage buffers must not overlap");
    static_assert(EPI_BYTES <= LDS_BYTES - SLOT, "the result staging area must stay clear of the other stage buffer");
    static_assert(LDS_BYTES + 64 <= 160 * 1024, "LDS budget");
};

// Swizzle: chunk position p of `row` holds logical chunk p ^ f(row); f makes the 16/CPR rows that share
// a 256-byte bank span use different positions.
template <int SB> __device__ __forceinline__ int swz(int row)
{
    constexpr int CPR = SB / 16;
    return (row / (16 / CPR)) % CPR;
}

// Chunk offsets (bytes inside a row block) a lane reads for MFMA step ks: FP8 two 16-byte chunks
// (bytes [16g,16g+16) and [32+16g, ...) of the step's 64-byte slab), FP4 one (bytes [16g, 16g+16) of
// the step's 32-byte slab).
template <int F, int SB, int KS>
__device__ __forceinline__ void frag_offsets(int r32, int g, int* off)
{
    const int f = swz<SB>(r32);          // row-block bases are multiples of 32 rows: f depends on r32 only
    constexpr int NC = F == kFP8 ? 2 * KS : KS;
#pragma unroll
    for (int k = 0; k < NC; ++k) {
        const int c = F == kFP8 ? ((k >> 1) * 4 + (k & 1) * 2 + g) : (k * 2 + g);
        off[k] = r32 * SB + ((c ^ f) * 16);
    }
}

template <int F>
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

// Dispatch id -> tile.  Workgroups are dealt round-robin to the 8 XCDs, so ids u, u + 8, u + 16, ... share an L2:
// each XCD gets a contiguous run of the tile sequence, and the sequence walks bands of 4 tile rows column by
// column, so that the 32 tiles an XCD works on at a time are a 4 x 8 patch (4 + 8 operand slabs for 32 tiles).
__device__ __forceinline__ void tile_of(int u, int nblk, int tiles_i, int tiles_j, int& ti, int& tj)
{
    int bid = u;
    const int per = nblk / 8;
    if (bid < per * 8) bid = (bid % 8) * per + bid / 8;
    const int band = 4;
    const int band_sz = band * tiles_j;
    const int b0 = bid / band_sz;
    const int rem = bid - b0 * band_sz;
    const int rows_in_band = min(band, tiles_i - b0 * band);
    ti = b0 * band + rem % rows_in_band;
    tj = rem / rows_in_band;
}

template <int FA, int FB, bool OUT_F32, class T>
__global__ __launch_bounds__(NT) void gemm_fast_kernel(const uint8_t* __restrict__ a_codes,
                                                       const uint8_t* __restrict__ a_g4,
                                                       const uint8_t* __restrict__ b_codes,
                                                       const uint8_t* __restrict__ b_g4,
                                                       int I, int J, int R, void* __restrict__ c_out, int64_t ldc,
                                                       int tiles_i, int tiles_j, float* __restrict__ norm_partials,
                                                       int stream_out)
{
    using C = FCfg<FA, FB, T>;
    constexpr int TM = T::TM, TN = T::TN, WTM = T::WTM, WTN = T::WTN, WGN = T::WGN, MB = T::MB, NB = T::NB;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[C::LDS_BYTES];
    // stage buffer layout: [A codes][B codes][A scale dwords: group-major, 256 rows][B scale dwords]

    const int nblk = tiles_i * tiles_j;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int r32 = lane & 31, g = lane >> 5;

    const int64_t a_row_bytes = FA == kFP8 ? R : R / 2;
    const int64_t b_row_bytes = FB == kFP8 ? R : R / 2;
    const int nstage = R / C::KE;                                     // >= 2 (gemm_fast_eligible)
    const int64_t a_pitch = g4_pitch(I), b_pitch = g4_pitch(J);      // dwords per scale group

    // ---- source addresses of the global->LDS copies of ONE tile (the tile the wave's copies currently belong
    //      to, which runs ahead of the tile being multiplied): wave-uniform base + per-lane 32-bit offset.
    //      Rows past the end of an operand re-read its last row (their products are never stored). ----
    unsigned oa[C::LA], ob[C::LB];
    const unsigned os = lane * 4;
    const uint8_t* sbase[C::LS];
    int64_t sstep[C::LS];
    const uint8_t* abase;
    const uint8_t* bbase;
    auto set_copy_tile = [&](int u) {
        int ti, tj;
        tile_of(u, nblk, tiles_i, tiles_j, ti, tj);
        const int i0 = ti * TM, j0 = tj * TN;
#pragma unroll
        for (int j = 0; j < C::LA; ++j) {
            constexpr int CPR = C::SBA / 16, RPI = 1024 / C::SBA;
            const int row = (wave * C::LA + j) * RPI + lane / CPR;
            const int c = (lane % CPR) ^ swz<C::SBA>(row);
            oa[j] = (unsigned)(min(row, I - 1 - i0) * a_row_bytes + c * 16);
        }
#pragma unroll
        for (int j = 0; j < C::LB; ++j) {
            constexpr int CPR = C::SBB / 16, RPI = 1024 / C::SBB;
            const int row = (wave * C::LB + j) * RPI + lane / CPR;
            const int c = (lane % CPR) ^ swz<C::SBB>(row);
            ob[j] = (unsigned)(min(row, J - 1 - j0) * b_row_bytes + c * 16);
        }
        // scale copy q of a stage: operand, scale group inside the stage, quarter of the 256 tile rows (the
        // padded pitch of the grouped copy covers whole tiles)
#pragma unroll
        for (int j = 0; j < C::LS; ++j) {
            const int q = wave * C::LS + j;
            const int opnd = q / (4 * C::NG), grp = (q % (4 * C::NG)) / 4;
            int quarter = q % 4;
            if (opnd == 1 && quarter * 64 >= TN) quarter -= TN / 64;      // a 128-row B tile: fetch its rows again (unused copy)
            const int64_t pitch = opnd == 0 ? a_pitch : b_pitch;
            sbase[j] = (opnd == 0 ? a_g4 : b_g4) + ((int64_t)grp * pitch + (opnd == 0 ? i0 : j0) + quarter * 64) * 4;
            sstep[j] = (int64_t)C::NG * pitch * 4;
        }
        abase = a_codes + (int64_t)i0 * a_row_bytes;
        bbase = b_codes + (int64_t)j0 * b_row_bytes;
    };
    const unsigned lds0 = lds_addr(lds);

    // all of this wave's copies of `stage` (of the copy tile) into stage buffer `slot`
    auto issue = [&](int stage, int slot) {
        const unsigned base = lds0 + slot * C::SLOT1;
#pragma unroll
        for (int j = 0; j < C::LA; ++j) glds16(abase + (int64_t)stage * C::SBA, oa[j], base + (wave * C::LA + j) * 1024);
#pragma unroll
        for (int j = 0; j < C::LB; ++j) glds16(bbase + (int64_t)stage * C::SBB, ob[j], base + C::A_BYTES + (wave * C::LB + j) * 1024);
#pragma unroll
        for (int j = 0; j < C::LS; ++j) glds4(sbase[j] + stage * sstep[j], os, base + C::A_BYTES + C::B_BYTES + (wave * C::LS + j) * 256);
    };
    // copy instruction j (0 .. L-1) of this wave's share of a stage
    auto issue_one = [&](int j, int stage, int slot) {
        const unsigned base = lds0 + slot * C::SLOT1;
        if (j < C::LA) glds16(abase + (int64_t)stage * C::SBA, oa[j], base + (wave * C::LA + j) * 1024);
        else if (j < C::LA + C::LB) { const int k = j - C::LA; glds16(bbase + (int64_t)stage * C::SBB, ob[k], base + C::A_BYTES + (wave * C::LB + k) * 1024); }
        else { const int k = j - C::LA - C::LB; glds4(sbase[k] + stage * sstep[k], os, base + C::A_BYTES + C::B_BYTES + (wave * C::LS + k) * 256); }
    };

    // ---- per-lane LDS read offsets ----
    constexpr int NCA = FA == kFP8 ? 2 * C::KS : C::KS, NCB = FB == kFP8 ? 2 * C::KS : C::KS;
    int offa[NCA], offb[NCB];
    frag_offsets<FA, C::SBA, C::KS>(r32, g, offa);
    frag_offsets<FB, C::SBB, C::KS>(r32, g, offb);
    const int sca_off = C::A_BYTES + C::B_BYTES + (wm * WTM + r32) * 4;
    const int scb_off = C::A_BYTES + C::B_BYTES + TM * C::NG * 4 + (wn * WTN + r32) * 4;

    v16f acc[MB][NB];

    // ---- ping-pong schedule.  The two waves that share a SIMD (wave w and w + 4) belong to different
    //      groups.  A stage is two phases; in every phase a wave either reads its operands of that phase
    //      from LDS into registers (R) or issues that phase's MFMAs (M).  Workgroup barriers separate the
    //      phases and group 1 runs one phase behind group 0, so while one wave of a SIMD feeds the matrix
    //      core the other one fetches:
    //          barrier    b0      b1      b2      b3      b4      b5 ...
    //          group 0        R0(0)   M0(0)   R1(0)   M1(0)   R0(1)   M0(1)
    //          group 1        -       R0(0)   M0(0)   R1(0)   M1(0)   R0(1)
    //      Stage s of a tile is complete in LDS before b(4s): every wave waits for its own copies before that
    //      barrier.  The buffer of stage s is free after b(4s+4): group 1, the last reader, waits for its R1(s)
    //      data before that barrier, so no read of the buffer is in flight when the first copy into it is issued.
    //      Stages alternate between the two buffers across tiles as well: stage s of a tile uses buffer
    //      (s + par) & 1, par being the number of stages of all earlier tiles mod 2.
    //      At the end of a tile (S stages): group 0 has issued its share of the next tile's stage 0 during
    //      M0(S-1) and group 1 during M1(S-2), both into the buffer that stage S would use.  After b(4S) group 0
    //      stores its result block through the staging area (which covers the last stage's buffer, free since
    //      b(4S)) while group 1 still issues M1(S-1), then group 1 stores its block; the next tile's b(0) follows.
    //      Group 1's share of the next tile's stage 1, which goes into the buffer under the staging area, is
    //      issued after that barrier (where the first tile issues it, too). ----
    constexpr int KP = C::KS / 2;                      // k-steps per phase
    v8i fa[KP][MB], fb[KP][NB];
    unsigned sa[MB], sb[NB];
    auto RD = [&](int slot, int p) {
        const uint8_t* base = lds + slot * C::SLOT1;
        const uint8_t* ta = base + wm * WTM * C::SBA;
        const uint8_t* tb = base + C::A_BYTES + wn * WTN * C::SBB;
        const int q = C::NG == 2 ? p : 0;
#pragma unroll
        for (int m = 0; m < MB; ++m) sa[m] = *reinterpret_cast<const unsigned*>(base + sca_off + q * TM * 4 + m * 128) >> (8 * g);
#pragma unroll
        for (int n = 0; n < NB; ++n) sb[n] = *reinterpret_cast<const unsigned*>(base + scb_off + q * TNP * 4 + n * 128) >> (8 * g);
#pragma unroll
        for (int k = 0; k < KP; ++k) {
#pragma unroll
            for (int m = 0; m < MB; ++m) fa[k][m] = read_frag<FA>(ta, m * 32 * C::SBA, offa, p * KP + k);
#pragma unroll
            for (int n = 0; n < NB; ++n) fb[k][n] = read_frag<FB>(tb, n * 32 * C::SBB, offb, p * KP + k);
        }
    };
    // The MFMAs of phase p.  With COPY the wave's L copy instructions of stage `nxt` (of the copy tile) into
    // buffer `nslot` are spread evenly between the phase's NM MFMAs (the sched_barriers keep them there).
    constexpr int NM = KP * MB * NB;
    auto MM = [&](auto copy_tag, int p, int nxt, int nslot) {
        constexpr bool COPY = decltype(copy_tag)::value;
        constexpr int ca = FB == kFP8 ? 0 : 4, cb = FA == kFP8 ? 0 : 4;
        __builtin_amdgcn_s_setprio(1);
        int idx = 0;
#pragma unroll
        for (int k = 0; k < KP; ++k) {
            const int ks = p * KP + k;
#pragma unroll
            for (int m = 0; m < MB; ++m)
#pragma unroll
                for (int n = 0; n < NB; ++n) {
                    if ((ks & 1) == 0)
                        acc[m][n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[k][n], fa[k][m], acc[m][n], ca, cb, 0, (int)sb[n], 0, (int)sa[m]);
                    else
                        acc[m][n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[k][n], fa[k][m], acc[m][n], ca, cb, 2, (int)sb[n], 2, (int)sa[m]);
                    if (COPY) {
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int j = 0; j < C::L; ++j)
                            if (j * NM / C::L == idx) issue_one(j, nxt, nslot);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    ++idx;
                }
        }
        __builtin_amdgcn_s_setprio(0);
    };
    const std::true_type with_copy{};
    const std::false_type no_copy{};
#define SNIP_BAR() do { __builtin_amdgcn_sched_barrier(0); __builtin_amdgcn_s_barrier(); __builtin_amdgcn_sched_barrier(0); } while (0)

    // ---- result of tile u: optional sum of squares, then every wave transposes its 128 x 64 block through its
    //      own 8 KB of the staging area at byte `ebase` of the LDS array ----
    auto store_tile = [&](int u, int ebase) {
        int ti, tj;
        tile_of(u, nblk, tiles_i, tiles_j, ti, tj);
        const int i0 = ti * TM, j0 = tj * TN;
        const bool interior = i0 + TM <= I && j0 + TN <= J;
        // optional: sum of squares of the tile as it will be stored (rounded to the output type), elements
        // outside the matrix excluded; one partial per tile, combined by a second kernel.  Interior tiles take
        // the short path: bf16 pairs are squared and added by v_dot2c_f32_bf16.
        if (norm_partials) {
            __shared__ float wave_ss[NWAVE];
            float ss = 0.f;
            if (interior) {
#pragma unroll
                for (int m = 0; m < MB; ++m)
#pragma unroll
                    for (int n = 0; n < NB; ++n)
#pragma unroll
                        for (int k = 0; k < 16; k += 2) {
                            if (OUT_F32) {
                                ss = fmaf(acc[m][n][k], acc[m][n][k], ss);
                                ss = fmaf(acc[m][n][k + 1], acc[m][n][k + 1], ss);
                            } else {
                                const float2_t pr = {acc[m][n][k], acc[m][n][k + 1]};
                                const bf16x2 r = __builtin_convertvector(pr, bf16x2);
                                const unsigned rb = __builtin_bit_cast(unsigned, r);
                                asm("v_dot2c_f32_bf16 %0, %1, %1" : "+v"(ss) : "v"(rb));       // ss += r.x * r.x + r.y * r.y
                            }
                        }
            } else {
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    const bool row_ok = i0 + wm * WTM + m * 32 + r32 < I;
#pragma unroll
                    for (int n = 0; n < NB; ++n)
#pragma unroll
                        for (int k = 0; k < 16; ++k) {
                            const int col = j0 + wn * WTN + n * 32 + 8 * (k >> 2) + 4 * g + (k & 3);
                            float v = acc[m][n][k];
                            if (!OUT_F32) v = (float)(__bf16)v;
                            ss = (row_ok && col < J) ? fmaf(v, v, ss) : ss;
                        }
                }
            }
            for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
            if (lane == 0) wave_ss[wave] = ss;
            __syncthreads();
            if (threadIdx.x == 0) {
                float t = 0.f;
                for (int w = 0; w < NWAVE; ++w) t += wave_ss[w];
                norm_partials[u] = t;
            }
        }
        // In registers, lane (r32, g) of block (m, n) holds C[32m + r32][32n + 8q + 4g + t] in acc[m][n][4q + t].
        // In LDS a row is ROWB bytes of 16-byte chunks, chunk c of row r stored at position c ^ f(r).
        constexpr int ESZ = OUT_F32 ? 4 : 2;
        constexpr int ROWB = WTN * ESZ;                  // 128 or 256 bytes per row
        constexpr int CPR = ROWB / 16;                   // 8 or 16 chunks per row
        constexpr int REGION = C::EPI_BYTES / NWAVE;     // LDS bytes a wave may use
        constexpr int ROWS_PER_PASS = REGION / ROWB < WTM ? REGION / ROWB : WTM;
        constexpr int MB_PER_PASS = ROWS_PER_PASS / 32;
        static_assert(MB_PER_PASS >= 1 && MB % MB_PER_PASS == 0, "staging passes must be whole 32-row blocks");
        uint8_t* reg = lds + ebase + wave * REGION;
#pragma unroll
        for (int pass = 0; pass < MB / MB_PER_PASS; ++pass) {
#pragma unroll
            for (int mm = 0; mm < MB_PER_PASS; ++mm) {
                const int m = pass * MB_PER_PASS + mm;
                const int row = mm * 32 + r32;
                const int f = OUT_F32 ? (row & (CPR - 1)) : ((row >> 1) & (CPR - 1));
#pragma unroll
                for (int n = 0; n < NB; ++n)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float v0 = acc[m][n][4 * q + 0], v1 = acc[m][n][4 * q + 1];
                        const float v2 = acc[m][n][4 * q + 2], v3 = acc[m][n][4 * q + 3];
                        if (OUT_F32) {
                            const int c = n * 8 + q * 2 + g;             // 4 floats = one chunk
                            *reinterpret_cast<float4*>(reg + row * ROWB + ((c ^ f) * 16)) = make_float4(v0, v1, v2, v3);
                        } else {
                            const int c = n * 4 + q;                     // 4 bf16 = half a chunk
                            const float2_t lo = {v0, v1}, hi = {v2, v3};
                            const bf16x2 blo = __builtin_convertvector(lo, bf16x2), bhi = __builtin_convertvector(hi, bf16x2);
                            *reinterpret_cast<uint2*>(reg + row * ROWB + ((c ^ f) * 16) + 8 * g) =
                                make_uint2(__builtin_bit_cast(unsigned, blo), __builtin_bit_cast(unsigned, bhi));
                        }
                    }
            }
            // read back row-contiguous: 64 lanes cover 64 / CPR rows per instruction.  All workgroups finish a tile
            // at about the same time: 32 MB per round of tiles, the size of all L2s together.  When operands and
            // output together fit the memory-side cache, plain stores are absorbed there fastest (2.1-2.7 us per tile
            // for the later group of waves against 3-5 us); when they do not, streaming stores keep the output from
            // pushing the operands out (8-10 % on the FP8 GEMMs with 180 MB operands).  The launcher decides.
            constexpr int RPI = 64 / CPR;
            if (interior) {
                // whole tile inside the matrix (wave-uniform): no per-lane tests, one wave-uniform base per
                // instruction plus a 32-bit lane offset
                const unsigned lane_off = (unsigned)((lane / CPR) * (int)ldc * ESZ + (lane % CPR) * 16);
                const uint8_t* cb = reinterpret_cast<const uint8_t*>(c_out) +
                                    ((int64_t)(i0 + wm * WTM + pass * ROWS_PER_PASS) * ldc + j0 + wn * WTN) * ESZ;
#pragma unroll
                for (int it = 0; it < ROWS_PER_PASS / RPI; ++it) {
                    const int row = it * RPI + lane / CPR;
                    const int c = lane % CPR;
                    const int f = OUT_F32 ? (row & (CPR - 1)) : ((row >> 1) & (CPR - 1));
                    const uint4 v = *reinterpret_cast<const uint4*>(reg + row * ROWB + ((c ^ f) * 16));
                    const v4u vv = {v.x, v.y, v.z, v.w};
                    uint8_t* p = const_cast<uint8_t*>(cb) + (int64_t)(it * RPI) * ldc * ESZ + lane_off;
                    if (stream_out) __builtin_nontemporal_store(vv, reinterpret_cast<v4u*>(p));
                    else *reinterpret_cast<v4u*>(p) = vv;
                }
            } else {
                for (int it = 0; it < ROWS_PER_PASS / RPI; ++it) {
                    const int row = it * RPI + lane / CPR;
                    const int c = lane % CPR;
                    const int f = OUT_F32 ? (row & (CPR - 1)) : ((row >> 1) & (CPR - 1));
                    const uint4 v = *reinterpret_cast<const uint4*>(reg + row * ROWB + ((c ^ f) * 16));
                    const int i = i0 + wm * WTM + pass * ROWS_PER_PASS + row;
                    const int j = j0 + wn * WTN + c * (16 / ESZ);
                    if (i < I) {
                        uint8_t* p = reinterpret_cast<uint8_t*>(c_out) + ((int64_t)i * ldc + j) * ESZ;
                        if (j + 16 / ESZ <= J) {
                            *reinterpret_cast<uint4*>(p) = v;
                        } else {
                            const unsigned w[4] = {v.x, v.y, v.z, v.w};
                            for (int e = 0; e < 16 / ESZ; ++e)
                                if (j + e < J) {
                                    if (OUT_F32) reinterpret_cast<unsigned*>(p)[e] = w[e];
                                    else reinterpret_cast<uint16_t*>(p)[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                                }
                        }
                    }
                }
            }
        }
    };

    int u = blockIdx.x;                  // dispatch id of the tile being multiplied
    int par = 0;                         // buffer of its stage 0
    bool first = true;
    set_copy_tile(u);
    issue(0, 0);
    for (;;) {
        const int un = u + (int)gridDim.x;
        const bool has_next = un < nblk;
#pragma unroll
        for (int a = 0; a < MB; ++a)
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int k = 0; k < 16; ++k) acc[a][b][k] = 0.f;
        const int ebase = ((nstage - 1 + par) & 1) ? C::LDS_BYTES - C::EPI_BYTES : 0;      // over the last stage's buffer
        if (wave < NWAVE / 2) {
            // group 0 issues its copies of stage s+1 during M0(s), between b(4s+1) and b(4s+2); during the last
            // stage these are the copies of the next tile's stage 0
            auto stage0 = [&](auto copy_tag, int s, int cstage) {
                const int slot = (s + par) & 1;
                // stage 0 of a later tile was waited for before the previous tile's result was stored; waiting
                // here again would wait for those stores
                if (s > 0 || first) SNIP_WAIT_VM(0);
                SNIP_BAR();                                         // b(4s)
                RD(slot, 0); SNIP_BAR();         // b(4s+1)
                MM(copy_tag, 0, cstage, slot ^ 1); SNIP_BAR();      // b(4s+2)
                RD(slot, 1); SNIP_BAR();         // b(4s+3)
                MM(no_copy, 1, 0, 0);
            };
            // Every stage carries copies, so that the MFMA code exists once (two variants of it merging in front
            // of the result store cost the register allocator its in-place accumulators).  Without a next tile the
            // last stage's copies re-fetch stage 0 of this tile into the free buffer, where nobody reads them.
            for (int s = 0; s < nstage; ++s) {
                const bool last = s == nstage - 1;
                if (last && has_next) set_copy_tile(un);
                stage0(with_copy, s, last ? 0 : s + 1);
            }
            SNIP_BAR();                                             // b(4S)
            SNIP_WAIT_VM(0);                                        // own share of the next tile's stage 0
        } else {
            // group 1 issues its copies of stage s+2 during M1(s), between b(4s+4) and b(4s+5) (during M1(S-2)
            // those of the next tile's stage 0, during M1(S-1) none); those of stage 1 while it idles through the
            // tile's first phase
            auto stage1 = [&](auto copy_tag, int s, int cstage) {
                const int slot = (s + par) & 1;
                SNIP_BAR();                                         // b(4s+1)
                RD(slot, 0); SNIP_BAR();         // b(4s+2)
                MM(no_copy, 0, 0, 0); SNIP_BAR();                   // b(4s+3)
                RD(slot, 1);
                __builtin_amdgcn_s_waitcnt(0x0070);                 // vmcnt(0) and lgkmcnt(0)
                SNIP_BAR();                                         // b(4s+4)
                MM(copy_tag, 1, cstage, slot);
            };
            if (first) SNIP_WAIT_VM(0);
            SNIP_BAR();                                             // b(0)
            issue(1, (1 + par) & 1);
            // (without a next tile the copies of M1(S-2) re-fetch stage 0 of this tile into the free buffer)
            for (int s = 0; s < nstage - 1; ++s) {
                const bool cross = s == nstage - 2;
                if (cross && has_next) set_copy_tile(un);
                stage1(with_copy, s, cross ? 0 : s + 2);
            }
            stage1(no_copy, nstage - 1, 0);
        }
        store_tile(u, ebase);
        if (!has_next) break;
        u = un;
        par = (par + nstage) & 1;
        first = false;
    }
#undef SNIP_BAR
}

// Compute units of the current device, a multiple of 8 (one share per XCD) so that dispatch ids u and u + grid
// land on the same XCD.
int compute_units()
{
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
        cached[dev] = n / 8 * 8;
    }
    return cached[dev];
}

// Which tile serves an I x J output best: the estimate is rounds of tiles over the compute units times the time of a
// tile; a 256 x 128 tile takes 0.6 of the time of a 256 x 256 one (half the MFMAs, three quarters of the operand bytes).
// The wide tile wins where the big one would leave compute units without a tile, or a last round nearly empty.
bool prefer_wide_tile(const GemmArgs& a)
{
    // SNIP_GEMM_TILE=big|wide in the environment fixes the tile (read at every call, so a test can cover both tiles
    // on every shape); anything else leaves the choice to the estimate below
    if (const char* e = getenv("SNIP_GEMM_TILE")) {
        if (e[0] == 'w') return true;
        if (e[0] == 'b') return false;
    }
    // A 256 x 128 tile costs about 0.8 of a 256 x 256 one (measured on one-round launches: per flop it reads more
    // of the LDS and stores as often), so it only pays while it fills compute units the larger tile would leave
    // idle, i.e. while it does not add a round of tiles.
    const int64_t ncu = compute_units();
    const int64_t big = ((a.I + 255) / 256) * ((a.J + 255) / 256), wide = ((a.I + 255) / 256) * ((a.J + 127) / 128);
    const double t_big = (double)((big + ncu - 1) / ncu), t_wide = 0.8 * (double)((wide + ncu - 1) / ncu);
    return t_wide < t_big;
}

template <int FA, int FB, class T>
hipError_t launch_fast_t(const GemmArgs& a, hipStream_t s)
{
    const int ti = (int)((a.I + T::TM - 1) / T::TM), tj = (int)((a.J + T::TN - 1) / T::TN);
    // one workgroup per compute unit (the LDS array admits no second one), each walking its share of the tiles
    const int ncu = compute_units();
    const dim3 grid((unsigned)(ti * tj < ncu ? ti * tj : ncu)), block(NT);
    // streaming output stores when operands + output exceed what the memory-side cache (256 MB) can hold next to
    // everything else in flight
    const double bytes = (double)a.I * a.R * (FA == kFP8 ? 1.0 : 0.5) + (double)a.J * a.R * (FB == kFP8 ? 1.0 : 0.5) +
                         (double)a.I * a.J * (a.out_fp32 ? 4.0 : 2.0);
    int stream_out = bytes > 200e6;
    if (a.out_fp32)
        hipLaunchKernelGGL((gemm_fast_kernel<FA, FB, true, T>), grid, block, 0, s, a.a_codes, a.a_scales_g4, a.b_codes, a.b_scales_g4,
                           (int)a.I, (int)a.J, (int)a.R, a.c, a.ldc, ti, tj, a.norm_partials, stream_out);
    else
        hipLaunchKernelGGL((gemm_fast_kernel<FA, FB, false, T>), grid, block, 0, s, a.a_codes, a.a_scales_g4, a.b_codes, a.b_scales_g4,
                           (int)a.I, (int)a.J, (int)a.R, a.c, a.ldc, ti, tj, a.norm_partials, stream_out);
    return hipGetLastError();
}

template <class T>
hipError_t launch_fast_tile(const GemmArgs& a, hipStream_t s)
{
    if (a.fmt_a == kFP8 && a.fmt_b == kFP8) return launch_fast_t<kFP8, kFP8, T>(a, s);
    if (a.fmt_a == kFP8 && a.fmt_b == kFP4) return launch_fast_t<kFP8, kFP4, T>(a, s);
    if (a.fmt_a == kFP4 && a.fmt_b == kFP8) return launch_fast_t<kFP4, kFP8, T>(a, s);
    return launch_fast_t<kFP4, kFP4, T>(a, s);
}

}  // namespace

bool gemm_fast_eligible(const GemmArgs& a)
{
    const int ke = (a.fmt_a == kFP4 && a.fmt_b == kFP4) ? 256 : 128;
    if (a.R > (1 << 22)) return false;      // per-lane source offsets are 32-bit: 256 rows x row bytes must fit
    return a.a_scales_g4 && a.b_scales_g4 && a.R % ke == 0 && a.R >= 2 * ke && a.I > 128 && a.J > 128;
}

int64_t gemm_fast_partials(const GemmArgs& a)
{
    return ((a.I + 255) / 256) * (prefer_wide_tile(a) ? (a.J + 127) / 128 : (a.J + 255) / 256);
}

hipError_t launch_gemm_fast(const GemmArgs& a, hipStream_t s)
{
    return prefer_wide_tile(a) ? launch_fast_tile<TileWide>(a, s) : launch_fast_tile<TileBig>(a, s);
}

}  // namespace snip
