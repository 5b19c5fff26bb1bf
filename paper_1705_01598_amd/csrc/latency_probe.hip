// Stand-alone latency probe for MI355X: measures the machine constants the analytical model of
// Section 2.3 needs (the paper obtains its own with a pointer-chasing benchmark and lists them
// in Table I): the latency of a dependent load as a function of the footprint it walks (vector
// L1, L2, memory-side cache, HBM), the LDS latency, and the departure delay -- the extra time
// each further independent request of one wave adds once the first is on its way.
//
//   latency_probe [max_footprint_mib]      (default 4096)
//
// Methods
//   chase:  one lane follows a random cycle through the 128-byte lines of a footprint (one
//           4-byte link per line, Sattolo's shuffle, so every line is visited once per lap and
//           no prefetcher or neighbouring-line effect helps); time per step = latency.
//   lds:    the same chase through a 32 KiB table in LDS.
//   burst:  one wave issues N independent wave-wide loads (64 lanes x 8 bytes = four lines
//           each) to lines nobody has touched since the caches were flushed, then waits for
//           all of them: T(N) = latency + (N - 1) * departure delay.
//   stream: one workgroup on one compute unit streams 256 MiB with 1, 4 or 8 loads in flight
//           per thread; bytes per cycle per compute unit.
// Time base: the constant-rate wall clock the kernels read (hipDeviceAttributeWallClockRate),
// converted to cycles of the published 2.4 GHz engine clock.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#define CHECK(call)                                                                           \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_));   \
            std::exit(1);                                                                     \
        }                                                                                     \
    } while (0)

namespace {

constexpr uint32_t kLineWords = 32;  // 128-byte line in 4-byte words
constexpr double kEngineGHz = 2.4;

// link[i] (one per line) is spread out so that line i of the footprint holds it in its first word
__global__ void spread_links_kernel(const uint32_t* __restrict__ link, uint32_t* __restrict__ lines, uint32_t n_lines) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_lines) lines[(size_t)i * kLineWords] = link[i];
}

// One lane: `warm` untimed dependent loads, then `steps` timed ones further along the same
// chain.  Every link is < n_lines by construction (checked on the host), so every access stays
// inside the footprint.  out[0] = wall-clock ticks, out[1] = the last position (keeps the chain
// alive).
__global__ void chase_kernel(const uint32_t* __restrict__ lines, uint32_t start, uint32_t warm, uint32_t steps, uint64_t* __restrict__ out) {
    uint32_t p = start;
    for (uint32_t i = 0; i < warm; ++i) {
        asm volatile("" : "+v"(p));  // keep the address in a vector register: a vector load
        p = lines[(size_t)p * kLineWords];
    }
    asm volatile("" : "+v"(p));
    const uint64_t t0 = wall_clock64();
    for (uint32_t i = 0; i < steps; ++i) {
        asm volatile("" : "+v"(p));
        p = lines[(size_t)p * kLineWords];
    }
    asm volatile("" : "+v"(p));
    const uint64_t t1 = wall_clock64();
    out[0] = t1 - t0;
    out[1] = p;
}

constexpr uint32_t kLdsWords = 8192;  // 32 KiB

__global__ void lds_chase_kernel(const uint32_t* __restrict__ link, uint32_t steps, uint64_t* __restrict__ out) {
    __shared__ uint32_t table[kLdsWords];
    for (uint32_t i = threadIdx.x; i < kLdsWords; i += blockDim.x) table[i] = link[i];
    __syncthreads();
    if (threadIdx.x != 0) return;
    uint32_t p = 0;
    const uint64_t t0 = wall_clock64();
    for (uint32_t i = 0; i < steps; ++i) {
        asm volatile("" : "+v"(p));
        p = table[p];
    }
    asm volatile("" : "+v"(p));
    const uint64_t t1 = wall_clock64();
    out[0] = t1 - t0;
    out[1] = p;
}

// One wave, N independent wave-wide loads of 512 bytes, request r at base + r * req_stride.
template <int N>
__global__ void __launch_bounds__(64) burst_kernel(const uint64_t* __restrict__ base, size_t req_stride_words, uint64_t* __restrict__ out) {
    typedef const __attribute__((address_space(1))) uint64_t* global_ptr;
    const uint64_t* q = base + threadIdx.x;
    uint64_t v[N];
    // the kernel's arguments have arrived before the clock is read: their own fetch is not timed
    asm volatile("" : "+v"(q), "+s"(req_stride_words));
    const global_ptr p = (global_ptr)q;  // still global memory (the register pass hid that from the compiler)
    const uint64_t t0 = wall_clock64();
#pragma unroll
    for (int r = 0; r < N; ++r) v[r] = __builtin_nontemporal_load(p + (size_t)r * req_stride_words);
#pragma unroll
    for (int r = 0; r < N; ++r) asm volatile("" : "+v"(v[r]));  // all values have arrived
    const uint64_t t1 = wall_clock64();
    uint64_t s = 0;
#pragma unroll
    for (int r = 0; r < N; ++r) s += v[r];
    if (threadIdx.x == 0) out[0] = t1 - t0;
    if (s == 0x123456789ull) out[1] = s;  // practically never true; keeps the loads
}

// One workgroup streams `n16` 16-byte words, every thread with U independent loads in flight
// (n16 is a multiple of U * blockDim.x); the sum keeps the loads.
typedef uint32_t word4 __attribute__((ext_vector_type(4)));

template <int U>
__global__ void __launch_bounds__(1024) stream_kernel(const word4* __restrict__ src, size_t n16, uint64_t* __restrict__ out) {
    uint32_t acc = 0;
    const size_t step = (size_t)U * blockDim.x;
    const uint64_t t0 = wall_clock64();
    for (size_t i = threadIdx.x; i < n16; i += step) {
        word4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + (size_t)u * blockDim.x);
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    asm volatile("" : "+v"(acc));
    __syncthreads();
    const uint64_t t1 = wall_clock64();
    if (threadIdx.x == 0) out[0] = t1 - t0;
    if (acc == 0x12345u) out[1] = acc;
}

double tick_ns = 10.0;

double to_cycles(double ns) { return ns * kEngineGHz; }

// Sattolo's algorithm: a uniformly random single cycle over n items
std::vector<uint32_t> random_cycle(uint32_t n, uint64_t seed) {
    std::vector<uint32_t> order(n);
    for (uint32_t i = 0; i < n; ++i) order[i] = i;
    std::mt19937_64 rng(seed);
    for (uint32_t i = n - 1; i > 0; --i) {
        const uint32_t j = (uint32_t)(rng() % i);
        std::swap(order[i], order[j]);
    }
    // order is a permutation that is one cycle when read as i -> order[i]
    return order;
}

bool is_valid_links(const std::vector<uint32_t>& link) {
    for (uint32_t v : link)
        if (v >= link.size()) return false;
    return true;
}

void flush_caches(void* scratch, size_t bytes) {
    CHECK(hipMemset(scratch, 0, bytes));
    CHECK(hipDeviceSynchronize());
}

template <int N>
double burst_ns(const uint64_t* region, size_t region_words, size_t req_stride_words, uint64_t* out_dev, int reps, size_t* cursor) {
    const size_t span = (size_t)(N - 1) * req_stride_words + 64;
    double total = 0;
    int done = 0;
    for (int i = 0; i < reps; ++i) {
        if (*cursor + span + 64 > region_words) break;  // fresh lines only
        hipLaunchKernelGGL(burst_kernel<N>, dim3(1), dim3(64), 0, 0, region + *cursor, req_stride_words, out_dev);
        CHECK(hipGetLastError());
        CHECK(hipDeviceSynchronize());
        uint64_t ticks = 0;
        CHECK(hipMemcpy(&ticks, out_dev, sizeof(ticks), hipMemcpyDeviceToHost));
        *cursor += span;  // the next repetition starts behind this one: untouched lines again
        if (i == 0) continue;  // the first launch of an instantiation loads its code
        total += (double)ticks * tick_ns;
        ++done;
    }
    return done ? total / done : -1.0;
}

}  // namespace

int main(int argc, char** argv) {
    size_t max_mib = 4096;
    if (argc > 1) max_mib = (size_t)std::strtoull(argv[1], nullptr, 10);
    if (max_mib < 1 || max_mib > 16384) {
        std::fprintf(stderr, "max_footprint_mib must be 1..16384\n");
        return 2;
    }
    int dev = 0;
    CHECK(hipSetDevice(dev));
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, dev));
    int wall_khz = 0;
    CHECK(hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, dev));
    if (wall_khz <= 0) {
        std::fprintf(stderr, "no wall clock rate reported\n");
        return 1;
    }
    tick_ns = 1.0e6 / (double)wall_khz;
    std::printf("device: %s (%s), %d compute units, engine clock %d MHz, wall clock %d kHz (tick %.1f ns)\n",
                prop.name[0] ? prop.name : "unnamed", prop.gcnArchName, prop.multiProcessorCount, prop.clockRate / 1000,
                wall_khz, tick_ns);
    std::printf("cycles below are at the published %.1f GHz engine clock\n\n", kEngineGHz);

    uint64_t* out_dev = nullptr;
    CHECK(hipMalloc(&out_dev, 2 * sizeof(uint64_t)));
    CHECK(hipMemset(out_dev, 0, 2 * sizeof(uint64_t)));

    void* flush = nullptr;
    const size_t flush_bytes = (size_t)1 << 30;  // larger than every cache level
    CHECK(hipMalloc(&flush, flush_bytes));

    // ---- chase through global memory ------------------------------------------------------
    // Up to 2^21 untimed steps first: one whole lap over footprints of up to 256 MiB, so the
    // timed steps find every line in the closest level that holds the footprint; beyond that
    // size the caches are flushed after the links are written and the timed steps run over
    // lines the walk has not seen, i.e. they come from HBM.
    std::printf("chase: dependent 4-byte vector loads, one per 128-byte line, random cycle over the footprint\n");
    std::printf("%12s %10s %10s %10s\n", "footprint", "steps", "ns/load", "cycles");
    const size_t max_bytes = max_mib << 20;
    uint32_t* lines = nullptr;
    CHECK(hipMalloc(&lines, max_bytes));
    CHECK(hipMemset(lines, 0, max_bytes));
    uint32_t* link_dev = nullptr;
    CHECK(hipMalloc(&link_dev, (max_bytes / 128) * sizeof(uint32_t)));
    for (size_t bytes = 4096; bytes <= max_bytes; bytes *= 4) {
        const uint32_t n_lines = (uint32_t)(bytes / 128);
        const std::vector<uint32_t> link = random_cycle(n_lines, 0x5eed0000ull + n_lines);
        if (!is_valid_links(link)) {
            std::fprintf(stderr, "bad link table\n");
            return 1;
        }
        CHECK(hipMemcpy(link_dev, link.data(), (size_t)n_lines * sizeof(uint32_t), hipMemcpyHostToDevice));
        hipLaunchKernelGGL(spread_links_kernel, dim3((n_lines + 255) / 256), dim3(256), 0, 0, link_dev, lines, n_lines);
        CHECK(hipGetLastError());
        CHECK(hipDeviceSynchronize());
        const bool beyond_caches = n_lines > (1u << 21);
        if (beyond_caches) flush_caches(flush, flush_bytes);
        const uint32_t warm = std::min<uint32_t>(std::max<uint32_t>(n_lines, 64u), 1u << 21);
        const uint32_t steps = std::min<uint32_t>(1u << 17, std::max<uint32_t>(n_lines * 4u, 4096u));
        hipLaunchKernelGGL(chase_kernel, dim3(1), dim3(1), 0, 0, lines, 0u, warm, steps, out_dev);
        CHECK(hipGetLastError());
        CHECK(hipDeviceSynchronize());
        uint64_t ticks = 0;
        CHECK(hipMemcpy(&ticks, out_dev, sizeof(ticks), hipMemcpyDeviceToHost));
        const double ns = (double)ticks * tick_ns / steps;
        char label[32];
        if (bytes >= ((size_t)1 << 20)) std::snprintf(label, sizeof label, "%zu MiB", bytes >> 20);
        else std::snprintf(label, sizeof label, "%zu KiB", bytes >> 10);
        std::printf("%12s %10u %10.1f %10.0f%s\n", label, steps, ns, to_cycles(ns), beyond_caches ? "   (unvisited lines after a flush)" : "");
        std::fflush(stdout);
    }

    // ---- chase through LDS ----------------------------------------------------------------
    {
        const std::vector<uint32_t> link = random_cycle(kLdsWords, 0x1d5ull);
        if (!is_valid_links(link)) return 1;
        CHECK(hipMemcpy(link_dev, link.data(), kLdsWords * sizeof(uint32_t), hipMemcpyHostToDevice));
        const uint32_t steps = 1u << 16;
        double best = 1e30;
        for (int rep = 0; rep < 3; ++rep) {
            hipLaunchKernelGGL(lds_chase_kernel, dim3(1), dim3(256), 0, 0, link_dev, steps, out_dev);
            CHECK(hipGetLastError());
            CHECK(hipDeviceSynchronize());
            uint64_t ticks = 0;
            CHECK(hipMemcpy(&ticks, out_dev, sizeof(ticks), hipMemcpyDeviceToHost));
            best = std::min(best, (double)ticks * tick_ns / steps);
        }
        std::printf("\nlds: dependent 4-byte loads from a 32 KiB table: %.1f ns = %.0f cycles\n", best, to_cycles(best));
        std::fflush(stdout);
    }

    // ---- burst: departure delay -----------------------------------------------------------
    {
        std::printf("\nburst: one wave, N independent wave-wide 512-byte loads to untouched lines, time until all have arrived\n");
        std::printf("%6s %12s %12s %22s\n", "N", "ns", "cycles", "cycles per extra request");
        const size_t region_bytes = std::min<size_t>(max_bytes, (size_t)512 << 20);
        const size_t region_words = region_bytes / 8;
        const size_t req_stride_words = (4096 + 512) / 8;  // requests 4.5 KiB apart: other lines, other channels
        flush_caches(flush, flush_bytes);
        const uint64_t* region = reinterpret_cast<const uint64_t*>(lines);
        size_t cursor = 0;
        const int reps = 33;
        double t1 = burst_ns<1>(region, region_words, req_stride_words, out_dev, reps, &cursor);
        struct Row { int n; double ns; } rows[6] = {{1, t1}, {2, 0}, {4, 0}, {8, 0}, {16, 0}, {32, 0}};
        rows[1].ns = burst_ns<2>(region, region_words, req_stride_words, out_dev, reps, &cursor);
        rows[2].ns = burst_ns<4>(region, region_words, req_stride_words, out_dev, reps, &cursor);
        rows[3].ns = burst_ns<8>(region, region_words, req_stride_words, out_dev, reps, &cursor);
        rows[4].ns = burst_ns<16>(region, region_words, req_stride_words, out_dev, reps, &cursor);
        rows[5].ns = burst_ns<32>(region, region_words, req_stride_words, out_dev, reps, &cursor);
        for (const Row& r : rows) {
            if (r.ns < 0) {
                std::printf("%6d %12s\n", r.n, "(region too small)");
                continue;
            }
            if (r.n == 1) std::printf("%6d %12.0f %12.0f %22s\n", r.n, r.ns, to_cycles(r.ns), "-");
            else std::printf("%6d %12.0f %12.0f %22.1f\n", r.n, r.ns, to_cycles(r.ns), to_cycles(r.ns - t1) / (r.n - 1));
        }
        std::printf("(a request is four 128-byte lines: divide by four for the delay per line)\n");
        std::fflush(stdout);
    }

    // ---- stream: what one compute unit can pull ---------------------------------------------
    {
        std::printf("\nstream: one workgroup on one compute unit reads 256 MiB with 16-byte nontemporal loads\n");
        std::printf("%8s %10s %12s %14s %16s\n", "threads", "in flight", "GB/s", "bytes/cycle", "cycles per line");
        const size_t bytes = std::min<size_t>(max_bytes, (size_t)256 << 20);
        for (int unroll : {1, 4, 8}) {
            for (int threads : {64, 256, 512, 1024}) {
                if ((bytes / 16) % ((size_t)unroll * threads) != 0) continue;
                double best = 1e30;
                for (int rep = 0; rep < 2; ++rep) {
                    const word4* src = reinterpret_cast<const word4*>(lines);
                    if (unroll == 1) hipLaunchKernelGGL(stream_kernel<1>, dim3(1), dim3(threads), 0, 0, src, bytes / 16, out_dev);
                    else if (unroll == 4) hipLaunchKernelGGL(stream_kernel<4>, dim3(1), dim3(threads), 0, 0, src, bytes / 16, out_dev);
                    else hipLaunchKernelGGL(stream_kernel<8>, dim3(1), dim3(threads), 0, 0, src, bytes / 16, out_dev);
                    CHECK(hipGetLastError());
                    CHECK(hipDeviceSynchronize());
                    uint64_t ticks = 0;
                    CHECK(hipMemcpy(&ticks, out_dev, sizeof(ticks), hipMemcpyDeviceToHost));
                    best = std::min(best, (double)ticks * tick_ns);
                }
                const double gbs = (double)bytes / best;
                const double bpc = gbs / kEngineGHz;
                char inflight[32];
                std::snprintf(inflight, sizeof inflight, "%d KiB", unroll * threads * 16 / 1024);
                std::printf("%8d %10s %12.1f %14.2f %16.1f\n", threads, inflight, gbs, bpc, 128.0 / bpc);
                std::fflush(stdout);
            }
        }
    }
    CHECK(hipFree(flush));
    CHECK(hipFree(link_dev));
    CHECK(hipFree(lines));
    CHECK(hipFree(out_dev));
    return 0;
}
