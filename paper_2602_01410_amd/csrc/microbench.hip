// Roofline denominators measured on the device: what the matrix cores, HBM and L2 actually deliver.
// Stand-alone program (built by build.py as snip_microbench, run by `bench.py --microbench`).
//   mfma   : v_mfma_scale_f32_32x32x64_f8f6f4 issue rate with constant operands (the datasheet figure) and
//            with random operands that change every instruction (what a GEMM on real data can reach: the
//            chip lowers its clock when the operand buses toggle)
//   copy   : streaming read+write of a buffer far larger than the 256 MB Infinity Cache (HBM)
//   l2     : every workgroup re-reads a 2 MB region with global->LDS copies (L2 hit bandwidth)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#include <cstdlib>
#include <string>
#include <vector>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(2);} } while (0)
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

template <int FMT, bool RANDOM>
__global__ __launch_bounds__(256) void k_mfma(const int* __restrict__ rnd, float* out, int iters)
{
    v8i a[4], b[4];
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 8; ++i) {
            const int ia = RANDOM ? (threadIdx.x * 8 + i + j * 2048) & 16383 : i;
            a[j][i] = rnd[ia];
            b[j][i] = rnd[(ia + 8192) & 16383];
            if (FMT == 0) { a[j][i] &= 0x77777777; b[j][i] &= 0x77777777; }     // keep FP8 codes finite
        }
    v16f acc[4];
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) acc[n][i] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 4; ++n)
            acc[n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[n], b[(n + 1) & 3], acc[n], FMT, FMT, 0, 120, 0, 120);
#pragma unroll
        for (int n = 0; n < 4; ++n)
            acc[n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[(n + 2) & 3], b[n], acc[n], FMT, FMT, 0, 120, 0, 120);
    }
    float s = 0;
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) s += acc[n][i];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void k_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void k_read(const uint4* __restrict__ src, size_t n, uint32_t* out)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    uint32_t acc = 0;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc += a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    if (acc == 0x9E3779B9u) out[0] = acc;       // keeps the loads alive
}

__global__ __launch_bounds__(512) void k_l2(const uint8_t* __restrict__ src, size_t region_bytes, int iters, uint32_t* out)
{
    __shared__ __attribute__((aligned(1024))) uint8_t buf[8 * 8 * 1024];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const unsigned base = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)buf + wave * 8192;
    size_t off = ((size_t)blockIdx.x * 7919 * 8192 + wave * 1024 + lane * 16) % region_bytes;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src + off), "s"(base + d * 1024) : "memory", "m0");
            off += 8192; if (off >= region_bytes) off -= region_bytes;
        }
        __builtin_amdgcn_s_waitcnt(0x0F70 | 4);      // vmcnt(4): keep half of them in flight
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    out[blockIdx.x * 512 + threadIdx.x] = ((uint32_t*)buf)[threadIdx.x];
}

// ---- sweep of streaming kernels: what HBM delivers for a copy, a pure read and a pure write as a function of
//      the launch shape (workgroups per compute unit), the loads a lane keeps in flight, the access width, the
//      walk (grid-stride, or one contiguous chunk per workgroup) and non-temporal hints ----
template <typename T, int U, bool NT, bool CHUNK>
__global__ __launch_bounds__(256) void k_stream(const T* __restrict__ src, T* __restrict__ dst, size_t n, int mode, uint32_t* sink)
{
    // mode 0: copy, 1: read only, 2: write only
    size_t i, stride, end;
    if (CHUNK) {
        const size_t per = (n + gridDim.x - 1) / gridDim.x;
        i = (size_t)blockIdx.x * per + threadIdx.x; stride = 256; end = (size_t)(blockIdx.x + 1) * per; if (end > n) end = n;
    } else {
        i = (size_t)blockIdx.x * 256 + threadIdx.x; stride = (size_t)gridDim.x * 256; end = n;
    }
    uint32_t acc = 0;
    T fill; __builtin_memset(&fill, 0x5A, sizeof(T));
    for (; i + (U - 1) * stride < end; i += U * stride) {
        T v[U];
        if (mode != 2) {
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = NT ? __builtin_nontemporal_load(src + i + u * stride) : src[i + u * stride];
        }
        if (mode == 1) {
#pragma unroll
            for (int u = 0; u < U; ++u) { const uint32_t* w = (const uint32_t*)&v[u]; for (unsigned k = 0; k < sizeof(T) / 4; ++k) acc ^= w[k]; }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const T o = mode == 0 ? v[u] : fill;
                if (NT) __builtin_nontemporal_store(o, dst + i + u * stride); else dst[i + u * stride] = o;
            }
        }
    }
    for (; i < end; i += stride) {
        if (mode == 1) { const T t = src[i]; const uint32_t* w = (const uint32_t*)&t; for (unsigned k = 0; k < sizeof(T) / 4; ++k) acc ^= w[k]; }
        else dst[i] = mode == 0 ? src[i] : fill;
    }
    if (mode == 1 && acc == 0x9E3779B9u) sink[0] = acc;
}

template <class F> float time_ms(F f, int reps)
{
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    f(); CK(hipDeviceSynchronize());
    CK(hipEventRecord(a));
    for (int i = 0; i < reps; ++i) f();
    CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b));
    return ms / reps;
}

typedef unsigned v4u __attribute__((ext_vector_type(4)));

template <typename T, int U, bool NT, bool CHUNK>
void sweep_one(const char* tag, const void* s, void* d, size_t bytes, uint32_t* sink)
{
    for (int wgpc : {1, 2, 4, 8, 16, 32}) {
        const int grid = wgpc * 256;
        double best[3];
        for (int mode = 0; mode < 3; ++mode) {
            const float ms = time_ms([&] { k_stream<T, U, NT, CHUNK><<<grid, 256>>>((const T*)s, (T*)d, bytes / sizeof(T), mode, sink); }, 3);
            best[mode] = (mode == 0 ? 2.0 : 1.0) * bytes / ms / 1e9;
        }
        printf("{\"kernel\": \"%s\", \"bytes_per_access\": %d, \"in_flight\": %d, \"nontemporal\": %d, \"walk\": \"%s\", \"wg_per_cu\": %d, "
               "\"copy_tbps\": %.2f, \"read_tbps\": %.2f, \"write_tbps\": %.2f}\n", tag, (int)sizeof(T), U, (int)NT,
               CHUNK ? "chunk" : "grid-stride", wgpc, best[0], best[1], best[2]);
        fflush(stdout);
    }
}

int hbm_sweep()
{
    const size_t bytes = 2048ull << 20;
    void *s, *d; CK(hipMalloc(&s, bytes)); CK(hipMalloc(&d, bytes)); CK(hipMemset(s, 1, bytes)); CK(hipMemset(d, 2, bytes));
    uint32_t* sink; CK(hipMalloc((void**)&sink, 64));
    {
        hipStream_t st; CK(hipStreamCreate(&st));
        const float ms = time_ms([&] { CK(hipMemcpyAsync(d, s, bytes, hipMemcpyDeviceToDevice, st)); CK(hipStreamSynchronize(st)); }, 5);
        printf("{\"kernel\": \"hipMemcpyAsync device-to-device\", \"copy_tbps\": %.2f}\n", 2.0 * bytes / ms / 1e9);
        const float ms2 = time_ms([&] { CK(hipMemsetAsync(d, 0, bytes, st)); CK(hipStreamSynchronize(st)); }, 5);
        printf("{\"kernel\": \"hipMemsetAsync\", \"write_tbps\": %.2f}\n", 1.0 * bytes / ms2 / 1e9);
    }
    sweep_one<v4u, 4, false, false>("stream", s, d, bytes, sink);
    sweep_one<v4u, 8, false, false>("stream", s, d, bytes, sink);
    sweep_one<v4u, 16, false, false>("stream", s, d, bytes, sink);
    sweep_one<v4u, 4, true, false>("stream", s, d, bytes, sink);
    sweep_one<v4u, 8, true, false>("stream", s, d, bytes, sink);
    sweep_one<v4u, 16, true, false>("stream", s, d, bytes, sink);
    sweep_one<v4u, 8, false, true>("stream", s, d, bytes, sink);
    sweep_one<v4u, 8, true, true>("stream", s, d, bytes, sink);
    sweep_one<unsigned, 8, false, false>("stream", s, d, bytes, sink);
    sweep_one<unsigned, 16, false, false>("stream", s, d, bytes, sink);
    sweep_one<unsigned, 16, true, false>("stream", s, d, bytes, sink);
    return 0;
}


// LDS read bandwidth: every lane of NW waves reads W-byte words, conflict-free (consecutive lanes, consecutive
// words), from a 64 KB array, UNR reads in flight per lane.
template <int W>
__global__ __launch_bounds__(512) void k_lds_read(int iters, uint32_t* out)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[65536];
    for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) ((uint32_t*)lds)[i] = i;
    __syncthreads();
    uint32_t acc = 0;
    unsigned off = threadIdx.x * W;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const unsigned a = (off + u * 8192) & 65535u;
            if (W == 16) { const uint4 v = *(const uint4*)(lds + a); acc ^= v.x ^ v.y ^ v.z ^ v.w; }
            else if (W == 8) { const uint2 v = *(const uint2*)(lds + a); acc ^= v.x ^ v.y; }
            else { acc ^= *(const uint32_t*)(lds + a); }
        }
        off += 1024;
    }
    if (acc == 0x12345678u) out[blockIdx.x] = acc;
}

static int lds_bench()
{
    uint32_t* out; CK(hipMalloc(&out, 4096 * 4));
    const int iters = 4000;
    printf("{");
    for (int nw : {4, 8}) {
        float ms;
        const double n = 1024.0 * nw * 64 * iters * 8;
        ms = time_ms([&] { k_lds_read<16><<<1024, nw * 64>>>(iters, out); }, 3);
        printf("\"lds_read_b128_%dwaves_tbps\": %.1f, ", nw, n * 16 / ms / 1e9);
        ms = time_ms([&] { k_lds_read<8><<<1024, nw * 64>>>(iters, out); }, 3);
        printf("\"lds_read_b64_%dwaves_tbps\": %.1f, ", nw, n * 8 / ms / 1e9);
        ms = time_ms([&] { k_lds_read<4><<<1024, nw * 64>>>(iters, out); }, 3);
        printf("\"lds_read_b32_%dwaves_tbps\": %.1f%s", nw, n * 4 / ms / 1e9, nw == 8 ? "" : ", ");
    }
    printf("}\n");
    return 0;
}

// MFMA issue rate with LDS reads going on beside it: every wave (8 per CU) issues 16 MFMAs on random operands that
// change every instruction, then READS ds_read_b128 of random LDS data, as a GEMM wave does per phase; the data read
// is only folded into a checksum.  Shows what the LDS -> register traffic of a tiling costs the matrix cores.
template <int FMT, int READS, int COPIES = 0>
__global__ __launch_bounds__(512) void k_mfma_lds(const int* __restrict__ rnd, float* out, int iters,
                                                  const uint8_t* __restrict__ src = nullptr, size_t region_bytes = 0)
{
    __shared__ __attribute__((aligned(1024))) uint8_t lds[65536 + (COPIES ? 65536 : 0)];
    for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) ((int*)lds)[i] = rnd[i & 16383];
    __syncthreads();
    v8i a[4], b[4];
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 8; ++i) {
            const int ia = (threadIdx.x * 8 + i + j * 2048) & 16383;
            a[j][i] = rnd[ia];
            b[j][i] = rnd[(ia + 8192) & 16383];
            if (FMT == 0) { a[j][i] &= 0x77777777; b[j][i] &= 0x77777777; }
        }
    v16f acc[4];
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) acc[n][i] = 0;
    unsigned chk = 0, off = (threadIdx.x & 63) * 16 + (threadIdx.x >> 6) * 1024;
    // COPIES global -> LDS copies of 1 KB per wave and iteration into a second 64 KB area, from a region that stays
    // in the memory-side caches (what a GEMM wave issues per phase for its share of the next stage)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned cbase = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)lds + 65536 + wave * 8192;
    size_t goff = COPIES ? ((size_t)blockIdx.x * 7919 * 8192 + wave * 1024 + (threadIdx.x & 63) * 16) % region_bytes : 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int n = 0; n < 4; ++n) {
                acc[n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[(n + r) & 3], b[(n + 2 * r + 1) & 3], acc[n], FMT, FMT, 0, 120, 0, 120);
                if (COPIES && (r * 4 + n) < COPIES) {
                    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src + goff), "s"(cbase + ((r * 4 + n) & 7) * 1024) : "memory", "m0");
                    goff += 8192; if (goff >= region_bytes) goff -= region_bytes;
                }
            }
        if (COPIES && (it & 1)) __builtin_amdgcn_s_waitcnt(0x0F70 | (COPIES < 15 ? COPIES : 15));   // at most one iteration's copies in flight
#pragma unroll
        for (int u = 0; u < READS; ++u) {
            const uint4 v = *(const uint4*)(lds + ((off + u * 8192) & 65535u));
            chk ^= v.x ^ v.y ^ v.z ^ v.w;
        }
        off += 1024;
    }
    if (COPIES) __builtin_amdgcn_s_waitcnt(0x0F70);
    float s = 0;
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) s += acc[n][i];
    out[blockIdx.x * 512 + threadIdx.x] = s + (chk == 0x12345678u ? 1.f : 0.f);
}

template <int FMT> static void mfma_lds_row(const int* rnd, float* out, const char* name, const uint8_t* src)
{
    const int iters = 4000;
    const double fl = 512.0 * 8 * iters * 16 * 2.0 * 32 * 32 * 64;
    float ms;
    ms = time_ms([&] { k_mfma_lds<FMT, 0><<<512, 512>>>(rnd, out, iters); }, 2);  printf("\"%s_reads0_tflops\": %.1f, ", name, fl / ms / 1e9);
    ms = time_ms([&] { k_mfma_lds<FMT, 4><<<512, 512>>>(rnd, out, iters); }, 2);  printf("\"%s_reads4_tflops\": %.1f, ", name, fl / ms / 1e9);
    ms = time_ms([&] { k_mfma_lds<FMT, 8><<<512, 512>>>(rnd, out, iters); }, 2);  printf("\"%s_reads8_tflops\": %.1f, ", name, fl / ms / 1e9);
    ms = time_ms([&] { k_mfma_lds<FMT, 12><<<512, 512>>>(rnd, out, iters); }, 2); printf("\"%s_reads12_tflops\": %.1f, ", name, fl / ms / 1e9);
    ms = time_ms([&] { k_mfma_lds<FMT, 24><<<512, 512>>>(rnd, out, iters); }, 2); printf("\"%s_reads24_tflops\": %.1f, ", name, fl / ms / 1e9);
    // the GEMM's own mix per wave and 16 MFMAs: FP4 12 reads + 5 copies, FP8 24 reads + 9 copies (codes and scales of a
    // 256 x 256 tile: 68 / 66 KB per stage over 8 waves); copies from a 2 MB region (L2 hits: the cheapest case)
    constexpr int R = FMT == 4 ? 12 : 24, C = FMT == 4 ? 5 : 9;
    ms = time_ms([&] { k_mfma_lds<FMT, R, C><<<512, 512>>>(rnd, out, iters, src, (size_t)2 << 20); }, 2);
    printf("\"%s_gemm_mix_reads%d_copies%d_tflops\": %.1f, ", name, R, C, fl / ms / 1e9);
    ms = time_ms([&] { k_mfma_lds<FMT, 0, C><<<512, 512>>>(rnd, out, iters, src, (size_t)2 << 20); }, 2);
    printf("\"%s_reads0_copies%d_tflops\": %.1f", name, C, fl / ms / 1e9);
}

static int mfma_lds_bench()
{
    int* rnd; CK(hipMalloc(&rnd, 16384 * 4));
    static int h[16384]; srand(1); for (int i = 0; i < 16384; ++i) h[i] = rand() ^ (rand() << 16);
    CK(hipMemcpy(rnd, h, sizeof h, hipMemcpyHostToDevice));
    float* out; CK(hipMalloc(&out, 512 * 512 * 4));
    uint8_t* src; CK(hipMalloc((void**)&src, (size_t)64 << 20));
    {   // random bytes in the copy source as well
        std::vector<int> big(((size_t)64 << 20) / 4);
        for (size_t i = 0; i < big.size(); ++i) big[i] = h[i & 16383] * (int)(2 * i + 1);
        CK(hipMemcpy(src, big.data(), (size_t)64 << 20, hipMemcpyHostToDevice));
    }
    printf("{");
    mfma_lds_row<4>(rnd, out, "fp4", src);
    printf(", ");
    mfma_lds_row<0>(rnd, out, "fp8", src);
    printf("}\n");
    return 0;
}

int main(int argc, char** argv)
{
    if (argc > 1 && std::string(argv[1]) == "mfma-lds") return mfma_lds_bench();
    if (argc > 1 && std::string(argv[1]) == "lds") return lds_bench();
    if (argc > 1 && std::string(argv[1]) == "hbm-sweep") return hbm_sweep();
    int* rnd; CK(hipMalloc(&rnd, 16384 * 4));
    static int h[16384]; srand(1); for (int i = 0; i < 16384; ++i) h[i] = rand() ^ (rand() << 16);
    CK(hipMemcpy(rnd, h, sizeof h, hipMemcpyHostToDevice));
    float* out; CK(hipMalloc(&out, 4096 * 512 * 4));
    const int iters = 20000;
    const double fl = 512.0 * 4 * iters * 8 * 2.0 * 32 * 32 * 64;
    printf("{");
    float ms;
    ms = time_ms([&] { k_mfma<4, false><<<512, 256>>>(rnd, out, iters); }, 2); printf("\"mfma_fp4_const_tflops\": %.1f, ", fl / ms / 1e9);
    ms = time_ms([&] { k_mfma<4, true><<<512, 256>>>(rnd, out, iters); }, 2);  printf("\"mfma_fp4_random_tflops\": %.1f, ", fl / ms / 1e9);
    ms = time_ms([&] { k_mfma<0, false><<<512, 256>>>(rnd, out, iters); }, 2); printf("\"mfma_fp8_const_tflops\": %.1f, ", fl / ms / 1e9);
    ms = time_ms([&] { k_mfma<0, true><<<512, 256>>>(rnd, out, iters); }, 2);  printf("\"mfma_fp8_random_tflops\": %.1f, ", fl / ms / 1e9);
    {
        const size_t bytes = 2048ull << 20;          // 2 GiB source + 2 GiB destination
        uint4 *s, *d; CK(hipMalloc((void**)&s, bytes)); CK(hipMalloc((void**)&d, bytes)); CK(hipMemset(s, 1, bytes));
        ms = time_ms([&] { k_copy<<<4096, 256>>>(s, d, bytes / 16); }, 5);
        printf("\"hbm_copy_read_plus_write_tbps\": %.2f, ", 2.0 * bytes / ms / 1e9);
        ms = time_ms([&] { k_read<<<4096, 256>>>(s, bytes / 16, (uint32_t*)out); }, 5);
        printf("\"hbm_read_only_tbps\": %.2f, ", 1.0 * bytes / ms / 1e9);
        ms = time_ms([&] { k_l2<<<256, 512>>>((const uint8_t*)s, 2u << 20, 400, (uint32_t*)out); }, 3);
        printf("\"l2_hit_read_tbps\": %.2f, ", 256.0 * 8 * 400 * 8 * 1024 / ms / 1e9);
        ms = time_ms([&] { k_l2<<<256, 512>>>((const uint8_t*)s, 64u << 20, 400, (uint32_t*)out); }, 3);
        printf("\"infinity_cache_read_tbps\": %.2f", 256.0 * 8 * 400 * 8 * 1024 / ms / 1e9);
    }
    printf("}\n");
    return 0;
}
