// Pattern probe (measurement tool, not part of the library): what does the memory system of
// an MI355X deliver for the global loads and stores of a 2-D transpose tile, whatever kernel
// issues them?
//
// A is an M x N matrix of 8-byte elements (M fastest), B its N x M transpose.  Persistent
// workgroups of 256 threads walk tiles of tm x tn elements and issue exactly the accesses a
// transposing tile kernel must: tn pieces of tm * 8 contiguous bytes read at pitch M * 8, tm
// pieces of tn * 8 bytes written at pitch N * 8, the next tile's loads issued with the current
// tile's stores.  The data take no transposing detour (the values land in the wrong places),
// so the rate is the ceiling that this access pattern allows; with lds = 1 every tile makes a
// conflict-free round trip through LDS between two barriers, the least a staged kernel pays.
//
// usage: pattern_probe M N  tm:tn:order:group:wgs:nt[:lds[:width]] ...
//   order  0 = tiles along M fastest (input-major), 1 = along N fastest (output-major),
//          w > 1 = windows of w tiles along M fastest, then along N, then the windows
//   group  255 = tiles in launch order, g = groups of 2^g consecutive tiles dealt to the 8 XCDs
//   wgs    workgroups per compute unit (grid = 256 * wgs)
//   nt     0 = cached loads and stores, 2 = nontemporal loads and stores
//   lds    0 / 1 (default 0);  width = bytes per lane and access, 16 or 8 (default 16)
// Tensors smaller than 256 MiB rotate through several places in 512 MiB buffers so that no
// launch finds its data in the last-level cache.  Prints one line per setting with the rate
// 2 * M * N * 8 / t in GB/s (1e9 bytes) over 8 (or 64) back-to-back launches.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int W> struct Access;
template <> struct Access<16> {
    typedef u32x4 t;
    template <int NT> static __device__ __forceinline__ t ld(__amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        return __builtin_amdgcn_raw_buffer_load_b128(r, (int)v, (int)s, NT);
    }
    template <int NT> static __device__ __forceinline__ void st(t x, __amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        __builtin_amdgcn_raw_buffer_store_b128(x, r, (int)v, (int)s, NT);
    }
};
template <> struct Access<8> {
    typedef u32x2 t;
    template <int NT> static __device__ __forceinline__ t ld(__amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        return __builtin_amdgcn_raw_buffer_load_b64(r, (int)v, (int)s, NT);
    }
    template <int NT> static __device__ __forceinline__ void st(t x, __amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        __builtin_amdgcn_raw_buffer_store_b64(x, r, (int)v, (int)s, NT);
    }
};

struct Params {
    uint32_t M, N, tm, tn, tiles_m, tiles_n, num_tiles, order, group_log2, nbytes;
};

__device__ __forceinline__ uint32_t tile_of(const Params& p, uint32_t block, uint32_t grid, uint32_t i) {
    if (p.group_log2 != 0xFFu) {
        const uint32_t xcd = block & 7u, slot = block >> 3, per = grid >> 3;
        const uint64_t local = (uint64_t)slot + (uint64_t)i * per;
        const uint64_t group = local >> p.group_log2;
        const uint64_t b = (((group << 3) + xcd) << p.group_log2) + (local & ((1u << p.group_log2) - 1u));
        return b < p.num_tiles ? (uint32_t)b : p.num_tiles;
    }
    const uint64_t b = (uint64_t)block + (uint64_t)i * grid;
    return b < p.num_tiles ? (uint32_t)b : p.num_tiles;
}

// Every access stays inside [0, nbytes): slot k of a tile reads piece k / pr < tn at 16- or 8-byte
// unit k % pr < pr of it, tiles tile the matrix exactly (M % tm == 0, N % tn == 0, checked on
// the host), and the buffer resource bounds the range in hardware besides.
template <int NREG, int NT, int LDS, int W>
__global__ void __launch_bounds__(256) pattern_kernel(const char* in, char* out, const Params p) {
    typedef typename Access<W>::t vt;
    extern __shared__ __align__(16) unsigned char smem[];
    vt* lds = reinterpret_cast<vt*>(smem);
    const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(in), 0, (int)p.nbytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(out, 0, (int)p.nbytes, 0x00020000);
    uint32_t rd[NREG], wr[NREG];
    const uint32_t pr = p.tm * 8 / W, pw = p.tn * 8 / W;  // access units per piece
#pragma unroll
    for (int s = 0; s < NREG; ++s) {
        const uint32_t k = s * 256 + threadIdx.x;
        rd[s] = ((k / pr) * p.M) * 8u + (k % pr) * W;
        wr[s] = ((k / pw) * p.N) * 8u + (k % pw) * W;
    }
    auto origin = [&](uint32_t t, uint32_t* oi, uint32_t* oo) {
        uint32_t ti, tj;
        if (p.order == 0) {
            ti = t % p.tiles_m;
            tj = t / p.tiles_m;
        } else if (p.order == 1) {
            tj = t % p.tiles_n;
            ti = t / p.tiles_n;
        } else {
            const uint32_t w = p.order, lo = t % w, r = t / w;
            tj = r % p.tiles_n;
            ti = (r / p.tiles_n) * w + lo;
        }
        *oi = (tj * p.tn * p.M + ti * p.tm) * 8u;
        *oo = (ti * p.tm * p.N + tj * p.tn) * 8u;
    };
    uint32_t it = 0;
    uint32_t t = tile_of(p, blockIdx.x, gridDim.x, it);
    vt v[NREG];
    uint32_t oi = 0, oo = 0;
    if (t < p.num_tiles) {
        origin(t, &oi, &oo);
#pragma unroll
        for (int s = 0; s < NREG; ++s) v[s] = Access<W>::template ld<NT>(rin, rd[s], oi);
    }
    while (t < p.num_tiles) {
        vt w[NREG];
        if (LDS) {
#pragma unroll
            for (int s = 0; s < NREG; ++s) lds[s * 256 + threadIdx.x] = v[s];
            __syncthreads();
#pragma unroll
            for (int s = 0; s < NREG; ++s) w[s] = lds[((s + 1) % NREG) * 256 + (threadIdx.x ^ 37u)];
        } else {
#pragma unroll
            for (int s = 0; s < NREG; ++s) w[s] = v[s];
        }
        const uint32_t next = tile_of(p, blockIdx.x, gridDim.x, ++it);
        uint32_t noi = 0, noo = 0;
#pragma unroll
        for (int s = 0; s < NREG; ++s) Access<W>::template st<NT>(w[s], rout, wr[s], oo);
        if (next < p.num_tiles) {
            origin(next, &noi, &noo);
#pragma unroll
            for (int s = 0; s < NREG; ++s) v[s] = Access<W>::template ld<NT>(rin, rd[s], noi);
        }
        t = next;
        oi = noi;
        oo = noo;
        if (LDS) __syncthreads();  // all waves are done with the image (every wave reaches it: t is uniform)
    }
}

typedef void (*kernel_t)(const char*, char*, const Params);
template <int NT, int LDS, int W> static kernel_t pick(int nreg) {
    switch (nreg) {
#define CASE(N) case N: return pattern_kernel<N, NT, LDS, W>;
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(6) CASE(8) CASE(12) CASE(16) CASE(24) CASE(32)
#undef CASE
    }
    return nullptr;
}

#define CHECK(x)                                                          \
    do {                                                                  \
        const hipError_t e_ = (x);                                        \
        if (e_ != hipSuccess) {                                           \
            std::printf("HIP error: %s (%s)\n", hipGetErrorString(e_), #x); \
            return 1;                                                     \
        }                                                                 \
    } while (0)

int main(int argc, char** argv) {
    if (argc < 4) {
        std::printf("usage: pattern_probe M N tm:tn:order:group:wgs:nt[:lds[:width]] ...\n");
        return 2;
    }
    const uint64_t M = std::strtoull(argv[1], nullptr, 10), N = std::strtoull(argv[2], nullptr, 10);
    const uint64_t nbytes = M * N * 8;
    if (M == 0 || N == 0 || nbytes >= ((uint64_t)1 << 32) - 256) {
        std::printf("M * N * 8 must be below 4 GiB\n");
        return 2;
    }
    const uint64_t places = nbytes >= (256u << 20) ? 1 : (512u << 20) / nbytes;
    char *a = nullptr, *b = nullptr;
    CHECK(hipMalloc(&a, nbytes * places));
    CHECK(hipMalloc(&b, nbytes * places));
    CHECK(hipMemset(a, 1, nbytes * places));
    CHECK(hipMemset(b, 0, nbytes * places));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int i = 3; i < argc; ++i) {
        unsigned tm, tn, order, group, wgs, nt, lds = 0, width = 16;
        if (std::sscanf(argv[i], "%u:%u:%u:%u:%u:%u:%u:%u", &tm, &tn, &order, &group, &wgs, &nt, &lds, &width) < 6 ||
            tm == 0 || tn == 0 || wgs == 0 || (width != 8 && width != 16) || (group != 255 && group > 16)) {
            std::printf("%s skipped (syntax)\n", argv[i]);
            continue;
        }
        const unsigned units = tm * tn * 8 / width;  // accesses per tile
        if (M % tm || N % tn || (tm * 8) % width || (tn * 8) % width || units % 256 ||
            (order > 1 && (M / tm) % order)) {
            std::printf("%s skipped (tiles must tile the matrix, pieces whole accesses, tile a multiple of 256 accesses)\n", argv[i]);
            continue;
        }
        const int nreg = (int)(units / 256);
        kernel_t k = width == 8 ? (lds ? (nt ? pick<2, 1, 8>(nreg) : pick<0, 1, 8>(nreg)) : (nt ? pick<2, 0, 8>(nreg) : pick<0, 0, 8>(nreg)))
                                : (lds ? (nt ? pick<2, 1, 16>(nreg) : pick<0, 1, 16>(nreg)) : (nt ? pick<2, 0, 16>(nreg) : pick<0, 0, 16>(nreg)));
        const size_t shmem = lds ? (size_t)nreg * 256 * width : 0;
        if (k == nullptr || shmem > 64 * 1024) {
            std::printf("%s skipped (%d accesses per thread not built, or LDS image above 64 KiB)\n", argv[i], nreg);
            continue;
        }
        Params p;
        p.M = (uint32_t)M; p.N = (uint32_t)N; p.tm = tm; p.tn = tn;
        p.tiles_m = (uint32_t)(M / tm); p.tiles_n = (uint32_t)(N / tn);
        p.num_tiles = p.tiles_m * p.tiles_n; p.order = order; p.group_log2 = group; p.nbytes = (uint32_t)nbytes;
        const int grid = 256 * (int)wgs;
        const int reps = places > 1 ? 64 : 8;
        auto launch = [&](int r) {
            const size_t off = (size_t)(r % places) * nbytes;
            hipLaunchKernelGGL(k, dim3(grid), dim3(256), shmem, 0, a + off, b + off, p);
        };
        for (int w = 0; w < 2; ++w) launch(w);
        CHECK(hipEventRecord(e0, 0));
        for (int r = 0; r < reps; ++r) launch(r);
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms = 0;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        std::printf("%-28s tile %ux%u read pieces %u B, written pieces %u B, tile %u KiB, %d x %u B per thread: %.0f GB/s\n",
                    argv[i], tm, tn, tm * 8, tn * 8, tm * tn * 8 / 1024, nreg, width, 2.0 * nbytes * reps / ms / 1e6);
        std::fflush(stdout);
    }
    CHECK(hipDeviceSynchronize());
    return 0;
}
