// Streaming microbenchmarks behind the access-shape choices of the update kernels: what one MI355X sustains on
// a 13 GB working set (the n = 128, d = 25.6 M model matrix of the headline configuration) for
//   - a read-only pass, a write-only pass and an out-of-place copy (the chip's plain streaming ceilings), and
//   - the in-place update of a round of disjoint row pairs,  avg = (x_i + x_j) / 2;  x_j <- avg;  x_i <- avg - c,
//     with 128-bit, 64-bit and 32-bit accesses per lane and 1 to 8 accesses per row in flight,
//   - an in-place triad (two reads, one write) traversed flat, by walking down the rows of a column tile, and by
//     one-tile blocks over 8 .. 128 far-apart pieces of the array,
// each as a kernel of its own name so that a kernel trace (rocprofv3 --kernel-trace --stats -- ./stream_bench)
// lists them side by side.  The program also times every kernel with HIP events and prints GB/s of algorithmic
// bytes.  Stand-alone: plain HIP runtime, no other file of the library.
//
//   stream_bench [rows (default 128)] [d (default 25600000)] [launches per kernel (default 10)]
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CHECK(expr)                                                                          \
    do {                                                                                     \
        hipError_t e__ = (expr);                                                             \
        if (e__ != hipSuccess) {                                                             \
            std::fprintf(stderr, "%s failed: %s\n", #expr, hipGetErrorString(e__));          \
            std::exit(1);                                                                    \
        }                                                                                    \
    } while (0)

namespace {

constexpr int kThreads = 256;

template <int VEC> struct Vec;
template <> struct Vec<1> { typedef float type; };
template <> struct Vec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct Vec<4> { typedef float type __attribute__((ext_vector_type(4))); };

struct Pair { int32_t i, j; };

// grid = (tiles of 256 * VEC * UNROLL floats, pairs).  Access u of thread t covers floats
// tile + (256 u + t) VEC .. + VEC - 1 of both rows: every wavefront instruction moves 64 VEC contiguous floats.
template <int VEC, int UNROLL>
__global__ __launch_bounds__(kThreads) void pair_update_kernel(float* X, int64_t ld, int64_t d, const Pair* pairs, float c) {
    typedef typename Vec<VEC>::type V;
    const Pair p = pairs[blockIdx.y];
    float* __restrict__ xi = X + static_cast<int64_t>(p.i) * ld;
    float* __restrict__ xj = X + static_cast<int64_t>(p.j) * ld;
    const int64_t e0 = (static_cast<int64_t>(blockIdx.x) * (kThreads * UNROLL) + threadIdx.x) * VEC;
    V a[UNROLL], b[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t e = e0 + static_cast<int64_t>(u) * kThreads * VEC;
        if (e < d) {
            a[u] = __builtin_nontemporal_load(reinterpret_cast<const V*>(xi + e));
            b[u] = __builtin_nontemporal_load(reinterpret_cast<const V*>(xj + e));
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t e = e0 + static_cast<int64_t>(u) * kThreads * VEC;
        if (e < d) {
            const V avg = (a[u] + b[u]) * 0.5f;
            __builtin_nontemporal_store(avg - c, reinterpret_cast<V*>(xi + e));
            __builtin_nontemporal_store(avg, reinterpret_cast<V*>(xj + e));
        }
    }
}

// read-only: grid-stride over 128-bit pieces, 8 loads in flight per lane, one partial per block
__global__ __launch_bounds__(kThreads) void read_only_kernel(const float* X, int64_t n_vec, float* partial) {
    typedef Vec<4>::type V;
    const V* src = reinterpret_cast<const V*>(X);
    float acc = 0.0f;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t v0 = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; v0 < n_vec; v0 += 8 * stride) {
        V x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = v0 + u * stride < n_vec ? __builtin_nontemporal_load(src + v0 + u * stride) : V{0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (x[u].x + x[u].y) + (x[u].z + x[u].w);
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((threadIdx.x & 63) == 0) atomicAdd(partial + blockIdx.x, acc);
}

// write-only: one 128-bit store per lane and step
__global__ __launch_bounds__(kThreads) void write_only_kernel(float* X, int64_t n_vec, float value) {
    typedef Vec<4>::type V;
    V* dst = reinterpret_cast<V*>(X);
    const V val = {value, value, value, value};
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; v < n_vec; v += stride)
        __builtin_nontemporal_store(val, dst + v);
}

// out-of-place copy, 4 x 128 bits in flight per lane
__global__ __launch_bounds__(kThreads) void copy_kernel(const float* src_f, float* dst_f, int64_t n_vec) {
    typedef Vec<4>::type V;
    const V* src = reinterpret_cast<const V*>(src_f);
    V* dst = reinterpret_cast<V*>(dst_f);
    const int64_t v0 = (static_cast<int64_t>(blockIdx.x) * 4) * kThreads + threadIdx.x;
    V x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (v0 + u * kThreads < n_vec) x[u] = __builtin_nontemporal_load(src + v0 + u * kThreads);
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (v0 + u * kThreads < n_vec) __builtin_nontemporal_store(x[u], dst + v0 + u * kThreads);
}

// In-place triad a <- a - c g (two reads and one write per element, the traffic of the synchronous mixing step with
// gradients from memory), in the two traversal orders an update kernel can have:
// flat: a block takes 1024 consecutive elements (one dword per lane, four in flight), the grid covers the array in order;
__global__ __launch_bounds__(kThreads) void triad_flat_kernel(float* A, const float* G, int64_t n, float c) {
    const int64_t e0 = static_cast<int64_t>(blockIdx.x) * (4 * kThreads) + threadIdx.x;
    float a[4], g[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t e = e0 + u * kThreads;
        if (e < n) {
            a[u] = __builtin_nontemporal_load(A + e);
            g[u] = __builtin_nontemporal_load(G + e);
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t e = e0 + u * kThreads;
        if (e < n) __builtin_nontemporal_store(a[u] - c * g[u], A + e);
    }
}
// row-walking: a block owns 1024 columns and walks down the rows, ROWS of them in flight (the order a kernel needs
// when the new row i depends on the old rows i - 1 and i + 1 and the update runs in place).
template <int ROWS>
__global__ __launch_bounds__(kThreads) void triad_rows_kernel(float* A, const float* G, int64_t ld, int64_t d, int rows, float c) {
    typedef Vec<4>::type V;
    const int64_t col = 4 * (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x);
    if (col >= d) return;
    for (int i0 = 0; i0 < rows; i0 += ROWS) {
        V a[ROWS], g[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
            if (i0 + r < rows) {
                a[r] = __builtin_nontemporal_load(reinterpret_cast<const V*>(A + static_cast<int64_t>(i0 + r) * ld + col));
                g[r] = __builtin_nontemporal_load(reinterpret_cast<const V*>(G + static_cast<int64_t>(i0 + r) * ld + col));
            }
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
            if (i0 + r < rows) __builtin_nontemporal_store(a[r] - c * g[r], reinterpret_cast<V*>(A + static_cast<int64_t>(i0 + r) * ld + col));
    }
}
// pieces: one-tile blocks (one 128-bit access per lane) over the array cut into PIECES equal contiguous pieces, the
// piece varying fastest with the block id: the chip then works on 2 x PIECES far-apart streams at a time.  Block ids go
// round the 8 XCDs, so with `rotate` off an XCD meets PIECES / 8 of the pieces (one, for 8) and with it on all of them.
__global__ __launch_bounds__(kThreads) void triad_pieces_kernel(float* A, const float* G, int64_t piece_len, int pieces, int rotate, float c) {
    typedef Vec<4>::type V;
    const int64_t tile = blockIdx.x / pieces;
    const int piece = static_cast<int>((blockIdx.x % pieces + (rotate ? tile : 0)) % pieces);
    const int64_t col = 4 * (tile * kThreads + threadIdx.x);
    if (col >= piece_len) return;
    const int64_t e = static_cast<int64_t>(piece) * piece_len + col;
    const V a = __builtin_nontemporal_load(reinterpret_cast<const V*>(A + e));
    const V g = __builtin_nontemporal_load(reinterpret_cast<const V*>(G + e));
    __builtin_nontemporal_store(a - c * g, reinterpret_cast<V*>(A + e));
}

struct Timer {
    hipEvent_t a, b;
    Timer() { CHECK(hipEventCreate(&a)); CHECK(hipEventCreate(&b)); }
    ~Timer() { (void)hipEventDestroy(a); (void)hipEventDestroy(b); }
};

template <typename Launch>
void measure(const char* name, double bytes, int launches, Launch&& launch) {
    Timer t;
    for (int w = 0; w < 2; ++w) launch();
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(t.a, nullptr));
    for (int r = 0; r < launches; ++r) launch();
    CHECK(hipEventRecord(t.b, nullptr));
    CHECK(hipEventSynchronize(t.b));
    CHECK(hipGetLastError());
    float ms = 0.0f;
    CHECK(hipEventElapsedTime(&ms, t.a, t.b));
    ms /= launches;
    std::printf("%-44s %9.3f ms  %8.1f GB/s  %5.1f %% of 8 TB/s\n", name, ms, bytes / (ms * 1e-3) / 1e9, bytes / (ms * 1e-3) / 8e12 * 100);
    std::fflush(stdout);
}

template <int VEC, int UNROLL>
void measure_pairs(float* X, int64_t ld, int64_t d, const Pair* pairs, int n_pairs, int launches) {
    char name[96];
    std::snprintf(name, sizeof name, "pair update in place, %3d-bit x %d in flight", 32 * VEC, UNROLL);
    const int64_t tile = static_cast<int64_t>(kThreads) * VEC * UNROLL;
    const dim3 grid(static_cast<uint32_t>((d + tile - 1) / tile), static_cast<uint32_t>(n_pairs));
    measure(name, 16.0 * d * n_pairs, launches, [&] {
        hipLaunchKernelGGL((pair_update_kernel<VEC, UNROLL>), grid, dim3(kThreads), 0, nullptr, X, ld, d, pairs, 1e-3f);
    });
}

}  // namespace

int main(int argc, char** argv) {
    const int rows = argc > 1 ? std::atoi(argv[1]) : 128;
    const int64_t d = argc > 2 ? std::atoll(argv[2]) : 25600000;
    const int launches = argc > 3 ? std::atoi(argv[3]) : 10;
    if (rows < 4 || rows > 4096 || (rows & 1) || d < 4 || (d & 3) || launches < 1 || launches > 1000) {
        std::fprintf(stderr, "usage: stream_bench [rows: even, 4..4096] [d: multiple of 4] [launches: 1..1000]\n");
        return 2;
    }
    const int64_t ld = d;
    const size_t bytes = static_cast<size_t>(rows) * ld * 4;
    size_t free_b = 0, total_b = 0;
    CHECK(hipMemGetInfo(&free_b, &total_b));
    if (bytes + (64u << 20) > free_b) {
        std::fprintf(stderr, "stream_bench: %zu bytes needed, %zu free\n", bytes, free_b);
        return 2;
    }
    float* X = nullptr;
    CHECK(hipMalloc(&X, bytes));
    const int blocks = 8192;
    float* partial = nullptr;
    CHECK(hipMalloc(&partial, blocks * sizeof(float)));
    CHECK(hipMemset(partial, 0, blocks * sizeof(float)));
    // a round of the ring schedule holds about 31 disjoint pairs: rows (4p, 4p + 1), p = 0 .. rows/4 - 1
    std::vector<Pair> host_pairs;
    for (int p = 0; 4 * p + 1 < rows && static_cast<int>(host_pairs.size()) < 31; ++p) host_pairs.push_back({4 * p, 4 * p + 1});
    const int n_pairs = static_cast<int>(host_pairs.size());
    Pair* pairs = nullptr;
    CHECK(hipMalloc(&pairs, n_pairs * sizeof(Pair)));
    CHECK(hipMemcpy(pairs, host_pairs.data(), n_pairs * sizeof(Pair), hipMemcpyHostToDevice));

    const int64_t n_vec = static_cast<int64_t>(rows) * ld / 4;
    std::printf("working set %d x %lld fp32 = %.2f GB; %d launches per kernel; %d pairs per update launch\n", rows,
                static_cast<long long>(d), bytes / 1e9, launches, n_pairs);
    measure("write only (128-bit stores)", static_cast<double>(bytes), launches, [&] {
        hipLaunchKernelGGL(write_only_kernel, dim3(blocks), dim3(kThreads), 0, nullptr, X, n_vec, 0.5f);
    });
    measure("read only (128-bit loads, 8 in flight)", static_cast<double>(bytes), launches, [&] {
        hipLaunchKernelGGL(read_only_kernel, dim3(blocks), dim3(kThreads), 0, nullptr, X, n_vec, partial);
    });
    const int64_t half_vec = n_vec / 2;
    measure("copy, first half -> second half (128-bit)", static_cast<double>(bytes), launches, [&] {
        hipLaunchKernelGGL(copy_kernel, dim3(static_cast<uint32_t>((half_vec + 4 * kThreads - 1) / (4 * kThreads))), dim3(kThreads), 0,
                           nullptr, X, X + half_vec * 4, half_vec);
    });
    measure_pairs<4, 1>(X, ld, d, pairs, n_pairs, launches);
    measure_pairs<4, 2>(X, ld, d, pairs, n_pairs, launches);
    measure_pairs<4, 4>(X, ld, d, pairs, n_pairs, launches);
    measure_pairs<2, 2>(X, ld, d, pairs, n_pairs, launches);
    measure_pairs<2, 4>(X, ld, d, pairs, n_pairs, launches);
    measure_pairs<1, 1>(X, ld, d, pairs, n_pairs, launches);
    measure_pairs<1, 2>(X, ld, d, pairs, n_pairs, launches);
    measure_pairs<1, 4>(X, ld, d, pairs, n_pairs, launches);
    measure_pairs<1, 8>(X, ld, d, pairs, n_pairs, launches);
    // triad: the first half of the rows is updated in place with the second half as its "gradient"
    {
        const int half = rows / 2;
        const int64_t n_half = static_cast<int64_t>(half) * ld;
        float* G = X + n_half;
        const double tbytes = 12.0 * n_half;
        measure("triad in place, flat (dword x 4)", tbytes, launches, [&] {
            hipLaunchKernelGGL(triad_flat_kernel, dim3(static_cast<uint32_t>((n_half + 4 * kThreads - 1) / (4 * kThreads))), dim3(kThreads), 0,
                               nullptr, X, G, n_half, 1e-3f);
        });
        const dim3 rgrid(static_cast<uint32_t>((d / 4 + kThreads - 1) / kThreads));
        measure("triad in place, row-walking, 2 rows in flight", tbytes, launches, [&] {
            hipLaunchKernelGGL(triad_rows_kernel<2>, rgrid, dim3(kThreads), 0, nullptr, X, G, ld, d, half, 1e-3f);
        });
        measure("triad in place, row-walking, 4 rows in flight", tbytes, launches, [&] {
            hipLaunchKernelGGL(triad_rows_kernel<4>, rgrid, dim3(kThreads), 0, nullptr, X, G, ld, d, half, 1e-3f);
        });
        measure("triad in place, row-walking, 8 rows in flight", tbytes, launches, [&] {
            hipLaunchKernelGGL(triad_rows_kernel<8>, rgrid, dim3(kThreads), 0, nullptr, X, G, ld, d, half, 1e-3f);
        });
        // what costs the row-walking order its bandwidth: the number of far-apart streams the chip, and each XCD, works on
        for (int rotate = 0; rotate < 2; ++rotate)
            for (int pieces : {8, 16, 32, 64, 128}) {
                if (n_half % (4 * static_cast<int64_t>(pieces)) != 0 || (rotate && pieces > 32)) continue;
                const int64_t piece_len = n_half / pieces;
                const int64_t tiles = (piece_len / 4 + kThreads - 1) / kThreads;
                if (tiles * pieces > 0x7fffffffLL) continue;
                char name[96];
                std::snprintf(name, sizeof name, "triad, one-tile blocks, %3d pieces%s", pieces, rotate ? ", rotated" : "");
                measure(name, tbytes, launches, [&] {
                    hipLaunchKernelGGL(triad_pieces_kernel, dim3(static_cast<uint32_t>(tiles * pieces)), dim3(kThreads), 0, nullptr, X, G, piece_len,
                                       pieces, rotate, 1e-3f);
                });
            }
    }
    CHECK(hipFree(pairs));
    CHECK(hipFree(partial));
    CHECK(hipFree(X));
    return 0;
}
