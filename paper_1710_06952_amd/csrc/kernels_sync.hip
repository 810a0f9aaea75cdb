// Synchronous comparison schedule: one iteration of decentralized parallel SGD
// as the related-work section of the paper describes it -- every worker averages
// its model with its neighbours while its gradient (taken at the model the
// iteration started from) is computed, then applies that gradient:
//     X[i] <- w_self[i] X[i] + sum_{j in N(i)} w_edge[i,j] X[j] - gamma g_i
// with a symmetric doubly stochastic weight matrix on the graph's edges.  With the
// experiments' optimizer (Sec. 5.2) the mixed model takes the place of the event's
// averaged model:  u = g_i + wd * mixed;  v_i <- mu v_i + u;  X[i] <- mixed - gamma v_i.
//
// Every column evolves independently of the others.  Iterations in pairs go to a second
// matrix and back with one-tile blocks in row order (the kernels at the end of this file);
// a single iteration runs in
// place: a block stages all n rows of a tile of 16..256 columns in LDS, then
// writes each row's mixture straight back to X.  HBM traffic is one
// read and one write of X (plus one read of the gradients for the data models, and a
// read and a write of the momentum buffers when they are in use).  When X exceeds the
// memory-side cache these streams bypass the caches (STREAM: non-temporal accesses; measured with
// gradients from slots on one box: 4.47 -> 4.60 TB/s at n = 128, d = 25.6 M and 4.45 -> 4.72 TB/s at
// n = 32, d = 4.2 M; for cache-resident sizes the plain accesses are up to 25 % faster, so they stay).
#include <algorithm>

#include "device_common.hpp"
#include "internal.hpp"

namespace adpsgd_impl {
namespace {

constexpr int kThreads = 256;

struct SyncParams {
    float* X;
    int64_t ld;
    int64_t d;
    int32_t n;
    int32_t cols;              // columns per block, a multiple of 4; cols / 4 divides kThreads
    const int32_t* rowptr;     // device copies of the graph and its weights
    const int32_t* col;
    const float* w_self;
    const float* w_edge;
    const float* slots;        // gradient of worker i in slot i (data models)
    uint16_t* Xbf16;
    float gamma;
    float synth_std;
    uint32_t key0, key1;
    uint64_t event0;           // synthetic gradients: worker i draws event event0 + i
    float* V;                  // momentum buffers (MOM), else nullptr
    float momentum, weight_decay;
    float* Y;                  // the ring written out of place: the matrix that receives the new models (same ld)
    int64_t tiles;             // ... its tiles of 1024 columns,
    uint32_t band;             // and the tiles per band of columns, a multiple of 8 (grid = (band, n, bands))
};

// grid = ceil(d / cols); thread = (quad of 4 columns, row lane)
// kBatch = rows of a thread whose global loads are issued together before the first use (a 16 KiB tile gives
// every thread four rows).  Measured on one box, 1 against 4: synthetic gradients at n = 128, d = 25.6 M
// 7.15 -> 6.47 ms; gradients from slots at n = 32, d = 4.2 M 4.73 -> 5.15 TB/s, but at n = 128 (32-column
// tiles) 4.63 -> 4.43 TB/s and for cache-resident models -7 %: the launcher picks per case.
template <bool SYNTH, bool SHADOW, bool MOM, bool STREAM, int kBatch>
__global__ __launch_bounds__(kThreads) void sync_mix_apply_kernel(const SyncParams p) {
    extern __shared__ __attribute__((aligned(16))) float tile[];   // [n][cols]
    const int quads = p.cols >> 2;
    const int qx = threadIdx.x % quads, ry = threadIdx.x / quads, rows_per_pass = kThreads / quads;
    const int64_t c = static_cast<int64_t>(blockIdx.x) * p.cols + 4 * qx;   // first of this thread's 4 columns
    const bool live = c < p.d;     // d is padded to a multiple of 4 by the leading dimension
    for (int r0 = ry; r0 < p.n; r0 += kBatch * rows_per_pass) {
        v4f v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int r = r0 + u * rows_per_pass;
            v[u] = v4f{0, 0, 0, 0};
            if (live && r < p.n) v[u] = load4<STREAM>(p.X + static_cast<int64_t>(r) * p.ld + c);
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int r = r0 + u * rows_per_pass;
            if (r < p.n) *reinterpret_cast<v4f*>(tile + static_cast<int64_t>(r) * p.cols + 4 * qx) = v[u];
        }
    }
    __syncthreads();
    if (!live) return;
    for (int i0 = ry; i0 < p.n; i0 += kBatch * rows_per_pass) {
        v4f g[kBatch], vo[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = i0 + u * rows_per_pass;
            g[u] = vo[u] = v4f{0, 0, 0, 0};
            if (i >= p.n) continue;
            if (SYNTH) {
                const uint64_t k = p.event0 + static_cast<uint64_t>(i);
                const uint64_t q = static_cast<uint64_t>(c) >> 2;
                g[u] = synth_normals4(static_cast<uint32_t>(q), static_cast<uint32_t>(q >> 32), static_cast<uint32_t>(k),
                                      static_cast<uint32_t>(k >> 32), p.key0, p.key1) * p.synth_std;
            } else {
                g[u] = load4<STREAM>(p.slots + static_cast<int64_t>(i) * p.ld + c);
            }
            if (MOM) vo[u] = load4<STREAM>(p.V + static_cast<int64_t>(i) * p.ld + c);
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = i0 + u * rows_per_pass;
            if (i >= p.n) continue;
            v4f acc = *reinterpret_cast<const v4f*>(tile + static_cast<int64_t>(i) * p.cols + 4 * qx) * p.w_self[i];
            const int32_t e1 = p.rowptr[i + 1];
            for (int32_t e = p.rowptr[i]; e < e1; ++e)
                acc += *reinterpret_cast<const v4f*>(tile + static_cast<int64_t>(p.col[e]) * p.cols + 4 * qx) * p.w_edge[e];
            v4f out;
            if (MOM) {
                const float mixed[4] = {acc.x, acc.y, acc.z, acc.w}, gv[4] = {g[u].x, g[u].y, g[u].z, g[u].w};
                const float vold[4] = {vo[u].x, vo[u].y, vo[u].z, vo[u].w};
                float xn[4], unused[4], vn[4];
#pragma unroll
                for (int t = 0; t < 4; ++t)      // the event's rule with both rows equal to the mixed model
                    average_then_apply_momentum(mixed[t], mixed[t], gv[t], vold[t], p.gamma, p.momentum, p.weight_decay,
                                                xn[t], unused[t], vn[t]);
                out = v4f{xn[0], xn[1], xn[2], xn[3]};
                v4f vout = {vn[0], vn[1], vn[2], vn[3]};
                if (c + 4 > p.d) {     // keep the padding beyond d at zero
                    if (c + 1 >= p.d) vout.y = 0.0f;
                    if (c + 2 >= p.d) vout.z = 0.0f;
                    if (c + 3 >= p.d) vout.w = 0.0f;
                }
                store4<STREAM>(p.V + static_cast<int64_t>(i) * p.ld + c, vout);
            } else {
#pragma clang fp contract(off)
                const v4f step = g[u] * p.gamma;
                out = acc - step;
            }
            if (c + 4 > p.d) {     // keep the padding beyond d at zero
                if (c + 1 >= p.d) out.y = 0.0f;
                if (c + 2 >= p.d) out.z = 0.0f;
                if (c + 3 >= p.d) out.w = 0.0f;
            }
            store4<STREAM>(p.X + static_cast<int64_t>(i) * p.ld + c, out);
            if (SHADOW) {
                v4h hb = {bf16_rne(out.x), bf16_rne(out.y), bf16_rne(out.z), bf16_rne(out.w)};
                *reinterpret_cast<v4h*>(p.Xbf16 + static_cast<int64_t>(i) * p.ld + c) = hb;
            }
        }
    }
}

// ---- the ring, without LDS -----------------------------------------------------------------------
// On a ring whose neighbour lists are in the canonical order (i - 1, i + 1) mod n, the mixture of row i
// needs rows i - 1, i and i + 1 only.  A thread that owns four columns walks down the rows with that
// three-row window in registers: every row is read once and written once by the same thread (row i is
// stored only after row i + 1 has been loaded; the old rows 0 and n - 1, which close the ring, are kept
// from the start), so the iteration runs in place without staging anything in LDS, and a block touches
// 4 KiB of every row instead of the 128-byte pieces the tile kernel is left with at n = 128.
// kRows rows are in flight per thread, whose four columns are one 128-bit piece.
// Measured on MI355X with gradients from slots (12 B per parameter and worker update: read X, read G, write X):
// n = 128, d = 25.6 M: 5.0-5.15 TB/s against 4.6 TB/s for the tile kernel; n = 32, d = 4.2 M: 4.5-5.5 TB/s
// against 4.9.  Nothing in the shape moves it: 2, 4 or 8 rows in flight, dwords or 128-bit pieces, blocks of
// 256, 512 or 1024 threads, a grid of one block per tile or 512-8192 blocks striding over the tiles all land
// within 3 % of each other.  The traversal binds: a plain in-place triad with the same two reads and one write
// per element streams 6.6 TB/s when the grid covers the arrays in order, and 5.3 TB/s when every block walks down
// the rows of its column tile, as a kernel must that updates in place when row i needs the old rows i - 1 and i + 1
// (stream_bench).  It runs an odd first iteration of a call, and every iteration when there is no second matrix;
// pairs of iterations take the kernel in row order below.
// The sums have the tile kernel's order (own row, then the neighbours as listed).
constexpr int kRingThreads = 256;
constexpr int kRingGridCap = 1024;

template <bool STREAM>
__device__ __forceinline__ void ring_load(const float* __restrict__ row, int64_t c, float out[4]) {
    const v4f v = load4<STREAM>(row + c);      // rows are padded to a multiple of 4 floats
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
template <bool STREAM>
__device__ __forceinline__ void ring_store(float* __restrict__ row, int64_t c, int64_t d, const float in[4]) {
    v4f v = {in[0], in[1], in[2], in[3]};
    if (c + 4 > d) {     // keep the padding beyond d at zero
        if (c + 1 >= d) v.y = 0.0f;
        if (c + 2 >= d) v.z = 0.0f;
        if (c + 3 >= d) v.w = 0.0f;
    }
    store4<STREAM>(row + c, v);
}

// grid: at most kRingGridCap blocks striding over the tiles of 1024 columns
template <bool SYNTH, bool SHADOW, bool MOM, bool STREAM, int kRows>
__global__ __launch_bounds__(kRingThreads) void sync_ring_apply_kernel(const SyncParams p) {
    const int32_t n = p.n;
    for (int64_t tile = blockIdx.x; tile * (4 * kRingThreads) < p.d; tile += gridDim.x) {
        const int64_t c = 4 * (tile * kRingThreads + threadIdx.x);
        if (c >= p.d) return;              // only in the last tile
        float first[4], prev[4], cur[4];
        ring_load<STREAM>(p.X, c, first);
        ring_load<STREAM>(p.X + static_cast<int64_t>(n - 1) * p.ld, c, prev);
#pragma unroll
        for (int t = 0; t < 4; ++t) cur[t] = first[t];
        for (int32_t i0 = 0; i0 < n; i0 += kRows) {
            float nxt[kRows][4], g[kRows][4], vo[kRows][4];
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                const int32_t i = i0 + u;
#pragma unroll
                for (int t = 0; t < 4; ++t) nxt[u][t] = first[t];          // row n is row 0, as it was
                if (i + 1 < n) ring_load<STREAM>(p.X + static_cast<int64_t>(i + 1) * p.ld, c, nxt[u]);
                if (i >= n) continue;
                if (SYNTH) {
                    const uint64_t k = p.event0 + static_cast<uint64_t>(i);
                    const uint64_t q = static_cast<uint64_t>(c) >> 2;
                    const v4f z = synth_normals4(static_cast<uint32_t>(q), static_cast<uint32_t>(q >> 32), static_cast<uint32_t>(k),
                                                 static_cast<uint32_t>(k >> 32), p.key0, p.key1) * p.synth_std;
                    g[u][0] = z.x; g[u][1] = z.y; g[u][2] = z.z; g[u][3] = z.w;
                } else {
                    ring_load<STREAM>(p.slots + static_cast<int64_t>(i) * p.ld, c, g[u]);
                }
                if (MOM) ring_load<STREAM>(p.V + static_cast<int64_t>(i) * p.ld, c, vo[u]);
            }
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                const int32_t i = i0 + u;
                if (i >= n) break;
                const float ws = p.w_self[i], wa = p.w_edge[2 * i], wb = p.w_edge[2 * i + 1];   // uniform: scalar loads
                float out[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    float acc = cur[t] * ws;
                    acc += prev[t] * wa;
                    acc += nxt[u][t] * wb;
                    if (MOM) {
                        float unused, vn;      // the event's rule with both rows equal to the mixed model
                        average_then_apply_momentum(acc, acc, g[u][t], vo[u][t], p.gamma, p.momentum, p.weight_decay, out[t], unused, vn);
                        vo[u][t] = vn;
                    } else {
#pragma clang fp contract(off)
                        const float step = g[u][t] * p.gamma;
                        out[t] = acc - step;
                    }
                }
                if (MOM) ring_store<STREAM>(p.V + static_cast<int64_t>(i) * p.ld, c, p.d, vo[u]);
                ring_store<STREAM>(p.X + static_cast<int64_t>(i) * p.ld, c, p.d, out);
                if (SHADOW) {
                    const v4h hb = {bf16_rne(out[0]), c + 1 < p.d ? bf16_rne(out[1]) : static_cast<uint16_t>(0),
                                    c + 2 < p.d ? bf16_rne(out[2]) : static_cast<uint16_t>(0),
                                    c + 3 < p.d ? bf16_rne(out[3]) : static_cast<uint16_t>(0)};
                    *reinterpret_cast<v4h*>(p.Xbf16 + static_cast<int64_t>(i) * p.ld + c) = hb;
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    prev[t] = cur[t];
                    cur[t] = nxt[u][t];
                }
            }
        }
    }
}

template <bool MOM, bool STREAM>
hipError_t launch_ring(const SyncParams& p, bool synth, hipStream_t st) {
    // a capped grid strides over the tiles of 1024 columns, every block the same number of them
    const int64_t tiles = (p.d + 4 * kRingThreads - 1) / (4 * kRingThreads);
    const int64_t passes = (tiles + kRingGridCap - 1) / kRingGridCap;
    const int64_t blocks = (tiles + passes - 1) / passes;
    const dim3 grid(static_cast<uint32_t>(blocks)), block(kRingThreads);
    if (synth) hipLaunchKernelGGL((sync_ring_apply_kernel<true, false, MOM, STREAM, 4>), grid, block, 0, st, p);
    else if (p.Xbf16) hipLaunchKernelGGL((sync_ring_apply_kernel<false, true, MOM, STREAM, 4>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((sync_ring_apply_kernel<false, false, MOM, STREAM, 4>), grid, block, 0, st, p);
    return hipGetLastError();
}

// ---- the ring, out of place, in row order ---------------------------------------------------------
// What holds the walking kernel at 5.0-5.15 TB/s is its traversal, not its code: with every block somewhere else
// on its way down the rows, the chip works on 2 x n far-apart address streams at a time and every XCD meets all
// of them; one-tile blocks over 128 far-apart pieces of an array lose the same bandwidth with no loop at all
// (stream_bench: 6.6 TB/s with 8 pieces, 5.0 with 128).  A traversal in row order cannot update in place, since
// the old row i is still needed by rows i - 1 and i + 1.  So iterations that come in pairs write the new models to
// a second matrix and back: a block is one tile of 1024 columns of ONE row (three loads of X, the gradient, one
// store per lane), and the grid (tile in band, row, band) is dispatched x fastest, i.e. in the order (band of ~2048
// tiles, row, tile).  The chip then works on about one
// row of a band at a time; tile t of rows i - 1, i, i + 1 meets the same XCD (block ids go round the 8 XCDs and the
// band widths are multiples of 8) 2048 and 4096 blocks apart, so two of the three loads of X hit that XCD's L2
// (a band of three rows is 24 MB of the chip's 32 MB) and HBM sees the same 12 B per parameter and worker update as
// in place (counters: 39.9 GB per iteration against 39.3 GB algorithmic).  Measured at n = 128, d = 25.6 M with
// gradients from slots: 6.84-6.93 ms per iteration = 5.7 TB/s against 7.7 ms in place; with momentum buffers 12.0
// against 13.1 ms; with gradients drawn in registers 5.3 against 6.0 ms.  A stand-alone kernel with this traversal
// and nothing else ran 6.54 ms with bands of 2048 tiles, 6.68 / 6.57 / 6.62 / 7.66 ms with 1024 / 1536 / 2560 / 3072;
// 7.3 / 7.6 ms with two / four rows per block (fewer loads through L2, more streams); 7.4 ms with one dword per lane
// and four accesses.  The loads of X stay cached whatever the size; the sums have the order of the walking kernel
// (own row, left, right), so both give the same bits.
constexpr uint32_t kBandTiles = 2048;

template <bool SYNTH, bool SHADOW, bool MOM, bool STREAM>
__global__ __launch_bounds__(kRingThreads) void sync_ring_rows_kernel(const SyncParams p) {
    const int32_t i = static_cast<int32_t>(blockIdx.y);     // blocks are dispatched x fastest: (band, row, tile) order
    const int64_t tile = static_cast<int64_t>(blockIdx.z) * p.band + blockIdx.x;
    const int64_t c = 4 * (tile * kRingThreads + threadIdx.x);
    if (tile >= p.tiles || c >= p.d) return;
    const int32_t im = i == 0 ? p.n - 1 : i - 1, ip = i == p.n - 1 ? 0 : i + 1;
    float prev[4], cur[4], nxt[4], g[4], vo[4];
    ring_load<false>(p.X + static_cast<int64_t>(ip) * p.ld, c, nxt);       // first touch of this tile: from HBM
    ring_load<false>(p.X + static_cast<int64_t>(i) * p.ld, c, cur);
    ring_load<false>(p.X + static_cast<int64_t>(im) * p.ld, c, prev);
    if (SYNTH) {
        const uint64_t k = p.event0 + static_cast<uint64_t>(i);
        const uint64_t q = static_cast<uint64_t>(c) >> 2;
        const v4f z = synth_normals4(static_cast<uint32_t>(q), static_cast<uint32_t>(q >> 32), static_cast<uint32_t>(k),
                                     static_cast<uint32_t>(k >> 32), p.key0, p.key1) * p.synth_std;
        g[0] = z.x; g[1] = z.y; g[2] = z.z; g[3] = z.w;
    } else {
        ring_load<STREAM>(p.slots + static_cast<int64_t>(i) * p.ld, c, g);
    }
    if (MOM) ring_load<STREAM>(p.V + static_cast<int64_t>(i) * p.ld, c, vo);
    const float ws = p.w_self[i], wa = p.w_edge[2 * i], wb = p.w_edge[2 * i + 1];   // uniform: scalar loads
    float out[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        float acc = cur[t] * ws;
        acc += prev[t] * wa;
        acc += nxt[t] * wb;
        if (MOM) {
            float unused, vn;      // the event's rule with both rows equal to the mixed model
            average_then_apply_momentum(acc, acc, g[t], vo[t], p.gamma, p.momentum, p.weight_decay, out[t], unused, vn);
            vo[t] = vn;
        } else {
#pragma clang fp contract(off)
            const float step = g[t] * p.gamma;
            out[t] = acc - step;
        }
    }
    if (MOM) ring_store<STREAM>(p.V + static_cast<int64_t>(i) * p.ld, c, p.d, vo);
    ring_store<STREAM>(p.Y + static_cast<int64_t>(i) * p.ld, c, p.d, out);
    if (SHADOW) {
        const v4h hb = {bf16_rne(out[0]), c + 1 < p.d ? bf16_rne(out[1]) : static_cast<uint16_t>(0),
                        c + 2 < p.d ? bf16_rne(out[2]) : static_cast<uint16_t>(0),
                        c + 3 < p.d ? bf16_rne(out[3]) : static_cast<uint16_t>(0)};
        *reinterpret_cast<v4h*>(p.Xbf16 + static_cast<int64_t>(i) * p.ld + c) = hb;
    }
}

// bands of one width of at most `limit` tiles, a multiple of 8 (the last band is cut short by at most 8 tiles per band
// in all: those blocks leave at once); false: the grid does not exist
bool rows_geometry(int32_t n, int64_t d, int64_t limit, int64_t& tiles, uint32_t& band, dim3& grid) {
    tiles = (d + 4 * kRingThreads - 1) / (4 * kRingThreads);
    if (n < 1 || n > 65535 || tiles < 1) return false;
    const int64_t want = (tiles + limit - 1) / limit;
    const int64_t width = ((tiles + want - 1) / want + 7) / 8 * 8;
    const int64_t count = (tiles + width - 1) / width;
    if (count > 65535) return false;
    band = static_cast<uint32_t>(width);
    grid = dim3(static_cast<uint32_t>(width), static_cast<uint32_t>(n), static_cast<uint32_t>(count));
    return true;
}
// tiles per band so that `rows` rows of a band stay in L2 (about 3 of the 4 MB of each of the 8 XCDs, 4 KiB per tile and row)
int64_t band_limit(int64_t rows) {
    const int64_t fit = (6144 / std::max<int64_t>(rows, 1)) / 8 * 8;
    return std::min<int64_t>(kBandTiles, std::max<int64_t>(fit, 8));
}

template <bool MOM, bool STREAM>
hipError_t launch_ring_rows(SyncParams& p, bool synth, hipStream_t st) {
    dim3 grid;
    const dim3 block(kRingThreads);
    if (p.n < 3 || !rows_geometry(p.n, p.d, band_limit(3), p.tiles, p.band, grid)) return hipErrorInvalidValue;
    if (synth) hipLaunchKernelGGL((sync_ring_rows_kernel<true, false, MOM, STREAM>), grid, block, 0, st, p);
    else if (p.Xbf16) hipLaunchKernelGGL((sync_ring_rows_kernel<false, true, MOM, STREAM>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((sync_ring_rows_kernel<false, false, MOM, STREAM>), grid, block, 0, st, p);
    return hipGetLastError();
}

// ---- any graph, out of place, in row order ----------------------------------------------------------
// The same traversal for a graph whose rows mix with arbitrary other rows: a block is one tile of one row and loads
// its own row and its neighbours' rows of X.  Any row may be needed again by any later row of the band, so the band
// is as wide as lets all n rows of it stay in L2 (48 tiles at n = 128): the first block that needs a row tile pulls it
// from HBM, the others find it in their XCD's L2.  Against the tile kernel this trades the LDS staging of 128-byte row
// pieces for 4 KiB pieces and L2 hits.  Measured at n = 128, d = 25.6 M, gradients from slots, per iteration: random
// 4-regular graph 9.06 ms in place (tile kernel), ring with the 2^i + 1 hop links (degree 16) 17.4 ms.
// The sum has the tile kernel's order: own row, then the neighbours as listed.
template <bool SYNTH, bool SHADOW, bool MOM, bool STREAM>
__global__ __launch_bounds__(kRingThreads) void sync_graph_rows_kernel(const SyncParams p) {
    const int32_t i = static_cast<int32_t>(blockIdx.y);     // blocks are dispatched x fastest: (band, row, tile) order
    const int64_t tile = static_cast<int64_t>(blockIdx.z) * p.band + blockIdx.x;
    const int64_t c = 4 * (tile * kRingThreads + threadIdx.x);
    if (tile >= p.tiles || c >= p.d) return;
    float own[4], g[4], vo[4];
    ring_load<false>(p.X + static_cast<int64_t>(i) * p.ld, c, own);
    if (SYNTH) {
        const uint64_t k = p.event0 + static_cast<uint64_t>(i);
        const uint64_t q = static_cast<uint64_t>(c) >> 2;
        const v4f z = synth_normals4(static_cast<uint32_t>(q), static_cast<uint32_t>(q >> 32), static_cast<uint32_t>(k),
                                     static_cast<uint32_t>(k >> 32), p.key0, p.key1) * p.synth_std;
        g[0] = z.x; g[1] = z.y; g[2] = z.z; g[3] = z.w;
    } else {
        ring_load<STREAM>(p.slots + static_cast<int64_t>(i) * p.ld, c, g);
    }
    if (MOM) ring_load<STREAM>(p.V + static_cast<int64_t>(i) * p.ld, c, vo);
    const float ws = p.w_self[i];
    float acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = own[t] * ws;
    const int32_t e1 = p.rowptr[i + 1];
    int32_t e = p.rowptr[i];
    for (; e + 4 <= e1; e += 4) {          // four neighbour rows in flight
        float nb[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) ring_load<false>(p.X + static_cast<int64_t>(p.col[e + u]) * p.ld, c, nb[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = p.w_edge[e + u];
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] += nb[u][t] * w;
        }
    }
    for (; e < e1; ++e) {
        float nb[4];
        ring_load<false>(p.X + static_cast<int64_t>(p.col[e]) * p.ld, c, nb);
        const float w = p.w_edge[e];
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] += nb[t] * w;
    }
    float out[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        if (MOM) {
            float unused, vn;      // the event's rule with both rows equal to the mixed model
            average_then_apply_momentum(acc[t], acc[t], g[t], vo[t], p.gamma, p.momentum, p.weight_decay, out[t], unused, vn);
            vo[t] = vn;
        } else {
#pragma clang fp contract(off)
            const float step = g[t] * p.gamma;
            out[t] = acc[t] - step;
        }
    }
    if (MOM) ring_store<STREAM>(p.V + static_cast<int64_t>(i) * p.ld, c, p.d, vo);
    ring_store<STREAM>(p.Y + static_cast<int64_t>(i) * p.ld, c, p.d, out);
    if (SHADOW) {
        const v4h hb = {bf16_rne(out[0]), c + 1 < p.d ? bf16_rne(out[1]) : static_cast<uint16_t>(0),
                        c + 2 < p.d ? bf16_rne(out[2]) : static_cast<uint16_t>(0),
                        c + 3 < p.d ? bf16_rne(out[3]) : static_cast<uint16_t>(0)};
        *reinterpret_cast<v4h*>(p.Xbf16 + static_cast<int64_t>(i) * p.ld + c) = hb;
    }
}

template <bool MOM, bool STREAM>
hipError_t launch_graph_rows(SyncParams& p, bool synth, hipStream_t st) {
    dim3 grid;
    const dim3 block(kRingThreads);
    if (!rows_geometry(p.n, p.d, band_limit(p.n), p.tiles, p.band, grid)) return hipErrorInvalidValue;
    if (synth) hipLaunchKernelGGL((sync_graph_rows_kernel<true, false, MOM, STREAM>), grid, block, 0, st, p);
    else if (p.Xbf16) hipLaunchKernelGGL((sync_graph_rows_kernel<false, true, MOM, STREAM>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((sync_graph_rows_kernel<false, false, MOM, STREAM>), grid, block, 0, st, p);
    return hipGetLastError();
}

template <bool MOM, bool STREAM>
hipError_t launch_variant(const SyncParams& p, bool synth, dim3 grid, size_t lds, hipStream_t st) {
    const bool wide = STREAM && p.cols >= 128;
    if (synth) hipLaunchKernelGGL((sync_mix_apply_kernel<true, false, MOM, STREAM, 4>), grid, dim3(kThreads), lds, st, p);
    else if (p.Xbf16 && wide) hipLaunchKernelGGL((sync_mix_apply_kernel<false, true, MOM, STREAM, 4>), grid, dim3(kThreads), lds, st, p);
    else if (p.Xbf16) hipLaunchKernelGGL((sync_mix_apply_kernel<false, true, MOM, STREAM, 1>), grid, dim3(kThreads), lds, st, p);
    else if (wide) hipLaunchKernelGGL((sync_mix_apply_kernel<false, false, MOM, STREAM, 4>), grid, dim3(kThreads), lds, st, p);
    else hipLaunchKernelGGL((sync_mix_apply_kernel<false, false, MOM, STREAM, 1>), grid, dim3(kThreads), lds, st, p);
    return hipGetLastError();
}

}  // namespace

int32_t sync_tile_cols(int32_t n) {
    // Widest tile of 16..256 columns whose n rows fit 16 KiB of LDS: several blocks then share a
    // compute unit and hide each other's latency (measured at n = 128, d = 25.6 M with synthetic
    // gradients: 7.2 ms per iteration with 16 KiB tiles, 9.9 ms with 32 KiB, 13.2 ms with 64 KiB).
    // More than 256 workers fall back to 16-column tiles of up to 64 KiB.
    constexpr int64_t kTileBytes = 16384;
    for (int32_t cols = 256; cols >= 16; cols >>= 1)
        if (static_cast<int64_t>(n) * cols * 4 <= kTileBytes) return cols;
    return static_cast<int64_t>(n) * 16 * 4 <= 65536 ? 16 : 0;
}

bool sync_out_of_place_ok(int32_t n, int64_t d) {
    int64_t tiles = 0;
    uint32_t band = 0;
    dim3 grid;
    return rows_geometry(n, d, band_limit(n), tiles, band, grid) && rows_geometry(n, d, band_limit(3), tiles, band, grid);
}

hipError_t launch_sync_mix_apply(const SyncArgs& a, hipStream_t st) {
    const int32_t cols = sync_tile_cols(a.n);
    if (cols == 0 || a.n < 1) return hipErrorInvalidValue;
    SyncParams p;
    p.X = a.X;
    p.ld = a.ld;
    p.d = a.d;
    p.n = a.n;
    p.cols = cols;
    p.rowptr = a.rowptr;
    p.col = a.col;
    p.w_self = a.w_self;
    p.w_edge = a.w_edge;
    p.slots = a.slots;
    p.Xbf16 = a.Xbf16;
    p.gamma = a.gamma;
    p.synth_std = a.synth_std;
    p.key0 = static_cast<uint32_t>(a.synth_seed);
    p.key1 = static_cast<uint32_t>(a.synth_seed >> 32);
    p.event0 = a.event0;
    const int64_t blocks = (a.d + cols - 1) / cols;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const size_t lds = static_cast<size_t>(a.n) * cols * 4;
    const dim3 grid(static_cast<uint32_t>(blocks));
    p.V = a.V;
    p.momentum = a.momentum;
    p.weight_decay = a.weight_decay;
    const bool stream = static_cast<int64_t>(a.n) * a.ld * 4 > (256ll << 20);      // X does not fit the memory-side cache
    p.Y = a.Xdst;
    p.tiles = 0;
    p.band = 0;
    if (a.Xdst) {
        if (a.Xdst == a.X) return hipErrorInvalidValue;
        if (a.ring) {
            if (stream) return a.V ? launch_ring_rows<true, true>(p, a.synth, st) : launch_ring_rows<false, true>(p, a.synth, st);
            return a.V ? launch_ring_rows<true, false>(p, a.synth, st) : launch_ring_rows<false, false>(p, a.synth, st);
        }
        if (stream) return a.V ? launch_graph_rows<true, true>(p, a.synth, st) : launch_graph_rows<false, true>(p, a.synth, st);
        return a.V ? launch_graph_rows<true, false>(p, a.synth, st) : launch_graph_rows<false, false>(p, a.synth, st);
    }
    if (a.ring) {
        if (stream) return a.V ? launch_ring<true, true>(p, a.synth, st) : launch_ring<false, true>(p, a.synth, st);
        return a.V ? launch_ring<true, false>(p, a.synth, st) : launch_ring<false, false>(p, a.synth, st);
    }
    if (stream) return a.V ? launch_variant<true, true>(p, a.synth, grid, lds, st) : launch_variant<false, true>(p, a.synth, grid, lds, st);
    return a.V ? launch_variant<true, false>(p, a.synth, grid, lds, st) : launch_variant<false, false>(p, a.synth, grid, lds, st);
}

}  // namespace adpsgd_impl
