// Attainable rates of the memory paths the executor could use, measured on the device it
// runs on (bench material, not part of the product path):
//   1. streaming a large array through the scalar data path (s_load) and through the
//      vector path (16-byte global loads);
//   2. gathering random rows of a small matrix with 4-, 8- and 16-byte loads per lane;
//   3. the same with the executor's access shape: every slice of a wave reads a
//      different row with 16-byte loads (rows of 512 / 256 / 128 bytes = 2 / 4 / 8 slices);
//   4. what a small launch costs: one workgroup of 8 waves per CU, launched back to back,
//      each wave following 0 to 4 dependent loads before it stores one word.
// hipEvent timing, best of 5 launches.  Build and run:
//   hipcc --offload-arch=gfx950 -O3 baselines/microbench_paths.hip -o microbench_paths && ./microbench_paths
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

typedef const uint32_t __attribute__((address_space(4))) cword_t;
#define CK(x)                                                                                  \
    do {                                                                                       \
        hipError_t e_ = (x);                                                                   \
        if (e_ != hipSuccess) {                                                                \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);             \
            exit(1);                                                                           \
        }                                                                                      \
    } while (0)

// ---- 1. streaming ---------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_scalar(const uint32_t *__restrict__ a, uint32_t words_per_wave,
                                                     uint32_t *out)
{
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const size_t w = (size_t)blockIdx.x * 4 + wave;
    cword_t *p = (cword_t *)a + w * words_per_wave;  // wave-uniform address: s_load
    uint32_t acc = 0;
    for (uint32_t i = 0; i < words_per_wave; i += 16) {
        uint32_t t[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) t[j] = p[i + j];
#pragma unroll
        for (int j = 0; j < 16; ++j) acc ^= t[j];
    }
    if ((threadIdx.x & 63) == 0) out[w] = acc;
}

__global__ __launch_bounds__(256) void stream_vector(const uint4 *__restrict__ a, uint32_t vec_per_wave, uint32_t *out)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t w = (size_t)blockIdx.x * 4 + wave;
    const uint4 *p = a + w * vec_per_wave;
    uint32_t acc = 0;
    for (uint32_t i = lane; i < vec_per_wave; i += 256) {
        const uint4 t0 = p[i], t1 = p[i + 64], t2 = p[i + 128], t3 = p[i + 192];
        acc ^= t0.x ^ t0.y ^ t0.z ^ t0.w ^ t1.x ^ t1.y ^ t1.z ^ t1.w ^ t2.x ^ t2.y ^ t2.z ^ t2.w ^ t3.x ^ t3.y ^ t3.z ^ t3.w;
    }
    out[w * 64 + lane] = acc;
}

// ---- 2. / 3. gathers --------------------------------------------------------------------
// LANES lanes read one row of LANES * VW floats with VW floats per lane; a wave holds
// 64 / LANES slices.  PER_SLICE: every slice draws its own row (the executor's shape);
// otherwise all slices read the same row.  U loads in flight per wave.
template <int VW, int LANES, int U, bool PER_SLICE>
__global__ __launch_bounds__(512) void gather(const float *__restrict__ B, uint32_t K, uint32_t iters, float *out)
{
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    const uint32_t id = (blockIdx.x * 8 + wave) * 64 + (PER_SLICE ? lane / LANES : 0);
    uint32_t s = id * 2654435761u + 12345u;
    const uint32_t ld = VW * LANES * 4;
    __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)B, 0, (int)(K * ld), 0x00020000);
    const uint32_t lo = (lane % LANES) * VW * 4;
    float acc = 0;
    for (uint32_t it = 0; it < iters; ++it) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            s = s * 1664525u + 1013904223u;
            const uint32_t off = lo + ((s >> 8) % K) * ld;
            if constexpr (VW == 1) {
                v[u] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, off, 0, 0));
            } else if constexpr (VW == 2) {
                auto t = __builtin_amdgcn_raw_buffer_load_b64(rs, off, 0, 0);
                v[u] = __uint_as_float(t[0] ^ t[1]);
            } else {
                auto t = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
                v[u] = __uint_as_float(t[0] ^ t[1] ^ t[2] ^ t[3]);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u];
    }
    out[(blockIdx.x * 8 + wave) * 64 + lane] = acc;
}

// ---- 4. launch cost and dependent loads -------------------------------------------------
template <int HOPS> __global__ __launch_bounds__(512) void chase(const uint32_t *__restrict__ table, uint32_t n, uint32_t *out)
{
    const uint32_t wave = blockIdx.x * 8 + (threadIdx.x >> 6);
    uint32_t at = (wave * 9973u + (threadIdx.x & 63u)) % n;
#pragma unroll
    for (int h = 0; h < HOPS; ++h) at = table[at];
    out[blockIdx.x * 512 + threadIdx.x] = at;
}

template <int HOPS> void run_chase(const uint32_t *table, uint32_t n, uint32_t *out, int groups)
{
    const int launches = 50;
    const float ms = best_ms([&] {
        for (int i = 0; i < launches; ++i) hipLaunchKernelGGL((chase<HOPS>), dim3(groups), dim3(512), 0, 0, table, n, out);
    });
    printf("launch of %d workgroups x 8 waves, %d dependent loads per wave: %5.2f us per launch (50 back to back)\n", groups,
           HOPS, ms * 1e3 / launches);
    fflush(stdout);
}

template <typename F> float best_ms(F f, int reps = 5)
{
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    f();
    CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int r = 0; r < reps; ++r) {
        CK(hipEventRecord(a));
        f();
        CK(hipEventRecord(b));
        CK(hipEventSynchronize(b));
        float ms;
        CK(hipEventElapsedTime(&ms, a, b));
        if (ms < best) best = ms;
    }
    CK(hipEventDestroy(a));
    CK(hipEventDestroy(b));
    return best;
}

template <int VW, int LANES, int U, bool PER_SLICE>
void run_gather(const char *what, const float *B, float *out, uint32_t K, int waves_per_cu, int cus, double ghz)
{
    const int waves = cus * waves_per_cu;
    const uint32_t iters = 4096 / U;
    const float ms = best_ms([&] {
        hipLaunchKernelGGL((gather<VW, LANES, U, PER_SLICE>), dim3(waves / 8), dim3(512), 0, 0, B, K, iters, out);
    });
    const double loads = (double)waves * iters * U;
    printf("%-34s row %3d B, B %5.2f MB, %2d waves/CU, %2d in flight: %6.2f G wave-loads/s, %5.1f TB/s moved, %5.1f clk/load/CU\n",
           what, VW * LANES * 4, (double)K * VW * LANES * 4 / 1e6, waves_per_cu, U, loads / ms / 1e6,
           loads * 64 * VW * 4 / ms / 1e9, cus * ghz * 1e9 / (loads / ms * 1e3));
    fflush(stdout);
}

int main()
{
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    const double ghz = prop.clockRate / 1e6;
    printf("%s: %d CUs, %.2f GHz\n", prop.gcnArchName, cus, ghz);

    const size_t bytes = 512ull << 20;
    uint32_t *a, *out;
    CK(hipMalloc(&a, bytes));
    CK(hipMemset(a, 1, bytes));
    CK(hipMalloc(&out, 64 << 20));
    for (int wpc : {4, 8, 16, 32}) {
        const int waves = cus * wpc;
        const uint32_t words = (uint32_t)((bytes / 4) / waves) & ~15u;
        float ms = best_ms([&] { hipLaunchKernelGGL(stream_scalar, dim3(waves / 4), dim3(256), 0, 0, a, words, out); });
        printf("stream, scalar loads, %2d waves/CU: %7.1f GB/s\n", wpc, (double)words * 4 * waves / ms / 1e6);
        const uint32_t vecs = (uint32_t)((bytes / 16) / waves) & ~255u;
        ms = best_ms([&] { hipLaunchKernelGGL(stream_vector, dim3(waves / 4), dim3(256), 0, 0, (const uint4 *)a, vecs, out); });
        printf("stream, 16-byte vector loads, %2d waves/CU: %7.1f GB/s\n", wpc, (double)vecs * 16 * waves / ms / 1e6);
        fflush(stdout);
    }

    float *B;
    CK(hipMalloc(&B, 64 << 20));
    CK(hipMemset(B, 0, 64 << 20));
    float *fo = (float *)out;
    printf("-- load width (all slices read the same random row)\n");
    run_gather<1, 64, 16, false>("4 B/lane, 64 lanes per row", B, fo, 2048, 32, cus, ghz);
    run_gather<2, 64, 16, false>("8 B/lane, 64 lanes per row", B, fo, 2048, 32, cus, ghz);
    run_gather<4, 32, 16, false>("16 B/lane, 2 x 32 lanes same row", B, fo, 2048, 32, cus, ghz);
    run_gather<2, 64, 16, false>("8 B/lane, 64 lanes per row", B, fo, 16384, 32, cus, ghz);
    run_gather<2, 64, 16, false>("8 B/lane, 64 lanes per row", B, fo, 131072, 32, cus, ghz);
    printf("-- the executor's shape: 16 B/lane, every slice its own random row\n");
    for (uint32_t K : {2048u, 8192u, 16384u}) {
        for (int wpc : {8, 16, 32}) {
            run_gather<4, 32, 8, true>("2 slices", B, fo, K, wpc, cus, ghz);
            run_gather<4, 32, 16, true>("2 slices", B, fo, K, wpc, cus, ghz);
            run_gather<4, 16, 8, true>("4 slices", B, fo, K, wpc, cus, ghz);
            run_gather<4, 8, 8, true>("8 slices", B, fo, K, wpc, cus, ghz);
        }
    }
    printf("-- small launches\n");
    {
        const uint32_t n = 1u << 20;
        uint32_t *host = (uint32_t *)malloc(n * 4), *table;
        for (uint32_t i = 0; i < n; ++i) host[i] = (uint32_t)(((uint64_t)i * 2654435761ull + 40503ull) % n);
        CK(hipMalloc(&table, n * 4));
        CK(hipMemcpy(table, host, n * 4, hipMemcpyHostToDevice));
        run_chase<0>(table, n, out, cus);
        run_chase<1>(table, n, out, cus);
        run_chase<2>(table, n, out, cus);
        run_chase<3>(table, n, out, cus);
        run_chase<4>(table, n, out, cus);
        for (int groups : {cus / 4, cus / 2, 2 * cus, 4 * cus, 8 * cus}) run_chase<3>(table, n, out, groups);
        free(host);
    }
    return 0;
}
