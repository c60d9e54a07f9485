// mxc_sweep — times template variants of the library's kernels on one GPU, so that the launch
// shapes chosen in mxc_dispatch.hpp can be re-checked (or re-tuned on other hardware).  Timing only: the
// inputs are pseudo-random bits, results are not inspected.
//
//   mxc_sweep [tokens] [hidden]        default 4096 8192, always 8 partials, block 32, E8M0 scale
//
// Besides the variants it times two probes that move the bytes of the 4-bit quantizer and of the
// 4-bit tile reduce in the same pattern without any arithmetic: the ceiling of each memory shape.
//
// Every variant is launched 20 times back to back over three rotating buffer sets (so that no
// launch reads what the previous one left in the last-level cache); the best of five such runs is
// printed as microseconds per launch, GB/s of algorithmic bytes and fraction of the 8 TB/s peak.
#include "mxc_kernels.hpp"

#include <cstdio>
#include <cstdlib>

using namespace mxc;

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(1);                                                              \
        }                                                                              \
    } while (0)

__global__ void fill_bits(uint32_t *p, size_t n, uint32_t seed, uint32_t and_mask, uint32_t or_mask)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i < n; i += (size_t)gridDim.x * blockDim.x) {
        uint32_t x = (uint32_t)i * 2654435761u ^ seed;
        x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
        p[i] = (x & and_mask) | or_mask;
    }
}

static size_t T = 4096, H = 8192, n, units;
static const int N = 8;
static hipEvent_t e0, e1;

template <class F>
static double best_ms(F launch)
{
    double best = 1e9;
    for (int k = 0; k < 5; ++k) {
        for (int i = 0; i < 3; ++i) launch(i);
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0, 0));
        const int reps = 20;
        for (int i = 0; i < reps; ++i) launch(i);
        CK(hipEventRecord(e1, 0));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        if (ms / reps < best) best = ms / reps;
    }
    return best;
}

static void report(const char *what, double ms, double bytes)
{
    std::printf("%-58s %8.1f us %8.1f GB/s  %.3f\n", what, ms * 1e3, bytes / ms / 1e6,
                bytes / ms / 1e6 / 8000.0);
    std::fflush(stdout);
}

struct Buffers {
    void *x[2][N];        // bf16 partials, two copies
    char *arena[3];       // packed sets, laid out as an all-gather would leave them
    void *out[3];         // binary32 tensors (reduce output / requantize input)
};
static Buffers b;
static const ScaleFmt sf{8, 127, 254, 255, 1};

static QuantArgs qargs(int i, int bits)
{
    QuantArgs a;
    const size_t cb = n * bits / 8, sb = n / 32;
    for (int r = 0; r < 32; ++r) {
        a.x[r] = b.x[i % 2][r % N];
        a.codes[r] = b.arena[i % 3] + (size_t)(r % N) * (cb + sb);
        a.scales[r] = b.arena[i % 3] + (size_t)(r % N) * (cb + sb) + cb;
    }
    a.units = units;
    a.sf = sf;
    return a;
}

static ReduceArgs rargs(int i, int bits)
{
    ReduceArgs a;
    const size_t cb = n * bits / 8, sb = n / 32;
    for (int r = 0; r < 32; ++r) {
        a.codes[r] = b.arena[i % 3] + (size_t)(r % N) * (cb + sb);
        a.scales[r] = b.arena[i % 3] + (size_t)(r % N) * (cb + sb) + cb;
    }
    a.out = b.out[i % 3];
    a.codes_out = a.scales_out = nullptr;
    a.own_x = nullptr;
    a.own_rank = -1;
    a.units = units;
    a.tp = N;
    a.sf = sf;
    return a;
}

template <int X, int Y, int U, bool NTL, bool NTS>
static void quant()
{
    const int bits = 1 + X + Y;
    const double ms = best_ms([&](int i) {
        QuantArgs a = qargs(i, bits);
        const unsigned g = (unsigned)((units + 256 * U - 1) / (256 * U));
        hipLaunchKernelGGL((quantize_kernel<Elem<X, Y>, 32, false, U, NTL, NTS, true>), dim3(g, N),
                           dim3(256), 0, 0, a);
    });
    char what[96];
    std::snprintf(what, sizeof what, "quantize bf16 e%dm%d  units/lane %d  nt loads %d  nt stores %d", X, Y, U,
                  (int)NTL, (int)NTS);
    report(what, ms, N * (n * 2.0 + n * bits / 8.0 + n / 32.0));
}

template <int X, int Y, int U, bool XPOSE>
static void quant32()
{
    const int bits = 1 + X + Y;
    const double ms = best_ms([&](int i) {
        QuantArgs a = qargs(i, bits);
        for (int r = 0; r < 32; ++r) a.x[r] = b.out[i % 3];
        const unsigned g = (unsigned)((units + 256 * U - 1) / (256 * U));
        hipLaunchKernelGGL((quantize_kernel<Elem<X, Y>, 32, true, U, true, true, true, XPOSE>), dim3(g, 1),
                           dim3(256), 0, 0, a);
    });
    char what[96];
    std::snprintf(what, sizeof what, "quantize f32  e%dm%d  units/lane %d  LDS-transposed loads %d", X, Y, U,
                  (int)XPOSE);
    report(what, ms, n * 4.0 + n * bits / 8.0 + n / 32.0);
}

template <int X, int Y, int RC, bool NTS>
static void reduce_unit()
{
    const int bits = 1 + X + Y;
    const double ms = best_ms([&](int i) {
        ReduceArgs a = rargs(i, bits);
        const unsigned g = (unsigned)((units + 256 * 4 - 1) / (256 * 4));
        hipLaunchKernelGGL((dequant_reduce_kernel<Elem<X, Y>, 32, false, 4, RC, true, NTS, true>), dim3(g),
                           dim3(256), 0, 0, a);
    });
    char what[96];
    std::snprintf(what, sizeof what, "reduce unit form e%dm%d  ranks together %d  nt stores %d", X, Y, RC, (int)NTS);
    report(what, ms, N * (n * bits / 8.0 + n / 32.0) + n * 4.0);
}

template <int X, int Y, int RC, bool NTS>
static void reduce_tile()
{
    const int bits = 1 + X + Y;
    const double ms = best_ms([&](int i) {
        ReduceArgs a = rargs(i, bits);
        const unsigned g = (unsigned)((units / 4 + 255) / 256);
        hipLaunchKernelGGL((dequant_reduce_tile_kernel<Elem<X, Y>, 32, false, RC, true, NTS, true>), dim3(g),
                           dim3(256), 0, 0, a);
    });
    char what[96];
    std::snprintf(what, sizeof what, "reduce tile form e%dm%d  ranks together %d  nt stores %d", X, Y, RC, (int)NTS);
    report(what, ms, N * (n * bits / 8.0 + n / 32.0) + n * 4.0);
}

template <int X, int Y, int RC, int WG>
static void reduce_tile_wg()
{
    const int bits = 1 + X + Y;
    const double ms = best_ms([&](int i) {
        ReduceArgs a = rargs(i, bits);
        const unsigned g = (unsigned)((units / 4 + WG - 1) / WG);
        hipLaunchKernelGGL((dequant_reduce_tile_kernel<Elem<X, Y>, 32, false, RC, true, true, true, false, false, WG>),
                           dim3(g), dim3(WG), 0, 0, a);
    });
    char what[96];
    std::snprintf(what, sizeof what, "reduce tile form e%dm%d  ranks together %d  nt stores 1  workgroup %d", X, Y, RC, WG);
    report(what, ms, N * (n * bits / 8.0 + n / 32.0) + n * 4.0);
}

template <int X, int Y, int RC>
static void fused()
{
    const int bits = 1 + X + Y;
    const double ms = best_ms([&](int i) {
        ReduceArgs a = rargs(i, bits);
        a.out = nullptr;
        a.codes_out = b.out[i % 3];
        a.scales_out = (char *)b.out[i % 3] + n;
        const unsigned g = (unsigned)((units / 4 + 255) / 256);
        hipLaunchKernelGGL((dequant_reduce_tile_kernel<Elem<X, Y>, 32, false, RC, true, true, true, true>),
                           dim3(g), dim3(256), 0, 0, a);
    });
    char what[96];
    std::snprintf(what, sizeof what, "fused reduce+requantize e%dm%d  ranks together %d", X, Y, RC);
    report(what, ms, (N + 1) * (n * bits / 8.0 + n / 32.0));
}

template <int U, bool NT>
static void copy()
{
    const size_t n16 = n * 4 / 16;
    const double ms = best_ms([&](int i) {
        const unsigned g = (unsigned)((n16 + 256 * U - 1) / (256 * U));
        hipLaunchKernelGGL((copy_kernel<U, NT>), dim3(g), dim3(256), 0, 0, (u32x4 *)b.out[i % 3],
                           (const u32x4 *)b.out[(i + 1) % 3], n16);
    });
    char what[96];
    std::snprintf(what, sizeof what, "copy  pieces/lane %d  nontemporal %d", U, (int)NT);
    report(what, ms, 2.0 * n * 4.0);
}


// Traffic of the 4-bit tile reduce without its arithmetic: per lane and rank one 16-byte code
// load and one scale byte, per lane eight 16-byte stores laid out as the reduce kernel's
// (contiguous 1 KiB per store instruction).  What it reaches is the ceiling of that memory
// shape on this GPU.
__global__ __launch_bounds__(256) void reduce_shape_probe(ReduceArgs a)
{
    const int lane = (int)(threadIdx.x & 63);
    const size_t tile = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const size_t chunk = tile * 64 + (size_t)lane;
    if (chunk >= a.units / 4) return;
    u32x4 c[8];
    uint32_t s = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        c[r] = __builtin_nontemporal_load((const u32x4 *)a.codes[r] + chunk);
        s += __builtin_nontemporal_load((const uint8_t *)a.scales[r] + chunk);
    }
    u32x4 *out = (u32x4 *)a.out + tile * 512;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        c[r].x ^= s;
        __builtin_nontemporal_store(c[r], out + r * 64 + lane);
    }
}

// Traffic of the 4-bit quantizer without its arithmetic: per lane a 16-byte bf16 load and a
// 4-byte store, one scale byte per four lanes, all eight partials in one launch.
__global__ __launch_bounds__(256) void quantize_shape_probe(QuantArgs a)
{
    const size_t unit0 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 2 - (threadIdx.x & 63);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const size_t unit = unit0 + (size_t)u * 64;
        if (unit >= a.units) continue;
        const u32x4 v = __builtin_nontemporal_load((const u32x4 *)a.x[blockIdx.y] + unit);
        const uint32_t w = v.x ^ v.y ^ v.z ^ v.w;
        __builtin_nontemporal_store(w, (uint32_t *)a.codes[blockIdx.y] + unit);
        if ((threadIdx.x & 3) == 0) ((uint8_t *)a.scales[blockIdx.y])[unit / 4] = (uint8_t)w;
    }
}

static void shape_probes()
{
    double ms = best_ms([&](int i) {
        ReduceArgs a = rargs(i, 4);
        hipLaunchKernelGGL(reduce_shape_probe, dim3((unsigned)((units / 4 + 255) / 256)), dim3(256), 0, 0, a);
    });
    report("traffic of the 4-bit tile reduce, no arithmetic", ms, N * (n / 2.0 + n / 32.0) + n * 4.0);
    ms = best_ms([&](int i) {
        QuantArgs a = qargs(i, 4);
        hipLaunchKernelGGL(quantize_shape_probe, dim3((unsigned)((units + 511) / 512), N), dim3(256), 0, 0, a);
    });
    report("traffic of the 4-bit quantizer, no arithmetic", ms, N * (n * 2.0 + n / 2.0 + n / 32.0));
}

int main(int argc, char **argv)
{
    if (argc > 1) T = (size_t)std::atoll(argv[1]);
    if (argc > 2) H = (size_t)std::atoll(argv[2]);
    if (T == 0 || H == 0 || (T * H) % 2048) {
        std::printf("tokens*hidden must be a positive multiple of 2048\n");
        return 1;
    }
    n = T * H;
    units = n / 8;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    for (int s = 0; s < 2; ++s)
        for (int r = 0; r < N; ++r) {
            CK(hipMalloc(&b.x[s][r], n * 2));
            // bf16 pairs with exponents around 1.0
            hipLaunchKernelGGL(fill_bits, dim3(4096), dim3(256), 0, 0, (uint32_t *)b.x[s][r], n / 2,
                               17u * r + s, 0x83FF83FFu, 0x3C003C00u);
        }
    const size_t set_bytes = (size_t)N * (n * 6 / 8 + n / 32);
    for (int s = 0; s < 3; ++s) {
        CK(hipMalloc(&b.arena[s], set_bytes));
        // bytes 0x70..0x7F everywhere (as scales: 2^-15..2^0); MXC_SWEEP_RANDOM_CODES=bits
        // overwrites the code regions of that code width with uniformly random bits
        hipLaunchKernelGGL(fill_bits, dim3(4096), dim3(256), 0, 0, (uint32_t *)b.arena[s], set_bytes / 4,
                           99u + s, 0x0F0F0F0Fu, 0x70707070u);
        if (const char *rb = std::getenv("MXC_SWEEP_RANDOM_CODES")) {
            const int bits = std::atoi(rb);
            const size_t cb = n * bits / 8, sb = n / 32;
            for (int r = 0; r < N; ++r)
                hipLaunchKernelGGL(fill_bits, dim3(4096), dim3(256), 0, 0,
                                   (uint32_t *)(b.arena[s] + (size_t)r * (cb + sb)), cb / 4, 7u * r + s,
                                   0xFFFFFFFFu, 0u);
        }
    }
    for (int s = 0; s < 3; ++s) {
        CK(hipMalloc(&b.out[s], n * 4));
        hipLaunchKernelGGL(fill_bits, dim3(4096), dim3(256), 0, 0, (uint32_t *)b.out[s], n, 5u + s,
                           0x83FFFFFFu, 0x3C000000u);
    }
    CK(hipDeviceSynchronize());
    std::printf("mxc_sweep: %d partials of [%zu x %zu], block 32, E8M0 scale\n", N, T, H);

    if (std::getenv("MXC_SWEEP_WG")) {
        reduce_tile_wg<2, 1, 4, 64>(); reduce_tile_wg<2, 1, 4, 128>(); reduce_tile_wg<2, 1, 4, 256>(); reduce_tile_wg<2, 1, 4, 512>();
        reduce_tile_wg<2, 2, 4, 64>(); reduce_tile_wg<2, 2, 4, 128>(); reduce_tile_wg<2, 2, 4, 256>();
        reduce_tile_wg<3, 2, 4, 64>(); reduce_tile_wg<3, 2, 4, 128>(); reduce_tile_wg<3, 2, 4, 256>();
        return 0;
    }
    copy<1, false>(); copy<4, false>(); copy<4, true>();
    shape_probes();
    quant<2, 1, 1, false, false>(); quant<2, 1, 2, false, false>(); quant<2, 1, 4, false, false>();
    quant<2, 1, 2, true, false>(); quant<2, 1, 1, true, true>(); quant<2, 1, 2, true, true>();
    quant<2, 1, 4, true, true>();
    quant<2, 2, 2, true, true>(); quant<2, 2, 4, true, true>();
    quant<3, 2, 2, true, true>(); quant<3, 2, 4, true, true>();
    quant32<2, 1, 1, false>(); quant32<2, 1, 2, false>(); quant32<2, 1, 1, true>(); quant32<2, 1, 2, true>();
    quant32<3, 2, 1, false>(); quant32<3, 2, 1, true>();
    reduce_unit<2, 1, 8, false>(); reduce_unit<2, 1, 8, true>();
    reduce_tile<2, 1, 4, false>();
    reduce_tile<2, 1, 2, true>(); reduce_tile<2, 1, 4, true>(); reduce_tile<2, 1, 8, true>();
    reduce_unit<2, 2, 8, true>();
    reduce_tile<2, 2, 2, false>();
    reduce_tile<2, 2, 2, true>(); reduce_tile<2, 2, 4, true>(); reduce_tile<2, 2, 8, true>();
    reduce_unit<3, 2, 8, true>();
    reduce_tile<3, 2, 4, false>();
    reduce_tile<3, 2, 2, true>(); reduce_tile<3, 2, 4, true>(); reduce_tile<3, 2, 8, true>();
    fused<2, 1, 4>(); fused<2, 1, 8>(); fused<2, 2, 8>(); fused<3, 2, 8>();
    return 0;
}
