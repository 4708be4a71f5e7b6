// Measured ceilings of one MI355X for the roofs the scoring kernels are priced against:
//   1. HBM read stream (what a kernel that only reads the feature matrix could reach);
//   2. LDS read throughput per compute unit for the access shapes of a tree visit
//      (an 8-byte node at a data-dependent address, a 4-byte feature in the lane's own bank),
//      with independent loads, so that issue rate and bank conflicts are measured, not latency;
//   3. a synthetic lock-step visit loop with the instruction sequence of the traversal kernel
//      (8 walks per lane, 12 wavefronts per compute unit, whole LDS), on random trees.
// Stand-alone program (not part of the library): `python -m paper_2201_00194_amd.build` builds
// it as fs_ceilings.bin next to the library; it prints a table and one JSON line.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x)                                                                       \
    do {                                                                            \
        hipError_t e_ = (x);                                                        \
        if (e_ != hipSuccess) {                                                     \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
            exit(1);                                                                \
        }                                                                           \
    } while (0)

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// UNROLL loads in flight per thread (1: the plain grid-stride loop).
template <int UNROLL>
__global__ void __launch_bounds__(512) stream_read_kernel(const u32x4 *__restrict__ p, size_t n16, uint32_t *out)
{
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    for (; i + (UNROLL - 1) * stride < n16; i += UNROLL * stride) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            v[u] = p[i + u * stride];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n16; i += stride) {
        const u32x4 a = p[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x12345678u)
        out[0] = acc;
}

// LDS read throughput.  Every lane keeps U byte addresses in registers; one iteration issues U
// independent reads (nothing depends on what comes back except a running xor).
//   WIDTH 4 / 8 / 16: ds_read_b32 / b64 / b128
enum Pattern {
    kLaneBank = 0,    // address = slot*256 + lane*WIDTH-stride: lane l stays in its own bank(s)
    kBroadcast = 1,   // all lanes the same address
    kRandomSmall = 2, // uniform over `span` bytes (a level of a tree: a few hundred bytes)
    kRandomAll = 3    // uniform over the whole buffer
};

// The reads are issued from inline assembly so that the compiler neither narrows, merges nor
// waits for them: nothing inside the loop consumes the destination registers; the hardware's
// own limit on outstanding LDS operations paces the loop.  The kernel has no static LDS, so
// byte addresses count from 0 of the dynamic block.
template <int WIDTH>
__device__ __forceinline__ void issue_read(uint32_t addr, u32x4 &dst)
{
#if defined(__HIP_DEVICE_COMPILE__)
    if (WIDTH == 2) {
        asm volatile("ds_read_u16 %0, %1" : "=v"(dst.x) : "v"(addr));
    } else if (WIDTH == 4) {
        asm volatile("ds_read_b32 %0, %1" : "=v"(dst.x) : "v"(addr));
    } else if (WIDTH == 8) {
        u32x2 t;
        asm volatile("ds_read_b64 %0, %1" : "=v"(t) : "v"(addr));
        dst.x = t.x;
        dst.y = t.y;
    } else {
        asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr));
    }
#else
    (void)addr; (void)dst;
#endif
}

template <int WIDTH, int U>
__global__ void __launch_bounds__(1024) lds_read_kernel(const uint32_t *__restrict__ addr_init, int lds_bytes,
                                                        int iters, uint32_t *out)
{
    extern __shared__ uint32_t lds[];
    for (int i = threadIdx.x; i < lds_bytes / 4; i += blockDim.x)
        lds[i] = (uint32_t)i * 2654435761u;
    __syncthreads();
    uint32_t a[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
        a[u] = addr_init[(size_t)u * blockDim.x + threadIdx.x];
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
        r[u] = u32x4{0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            issue_read<WIDTH>(a[u], r[u]);
    }
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#endif
    uint32_t acc = 0;
#pragma unroll
    for (int u = 0; u < U; ++u)
        acc ^= r[u].x ^ r[u].y ^ r[u].z ^ r[u].w;
    if (acc == 0x12345678u)
        out[0] = acc;
}

static uint32_t g_rng = 12345;
static uint32_t rnd()
{
    g_rng = g_rng * 1664525u + 1013904223u;
    return g_rng >> 8;
}

template <int WIDTH, int U>
static double run_lds(const char *name, Pattern pat, int waves, int lds_bytes, int span, int n_cu, uint32_t *d_out)
{
    const int threads = waves * 64;
    std::vector<uint32_t> h((size_t)U * threads);
    for (int u = 0; u < U; ++u)
        for (int t = 0; t < threads; ++t) {
            const int lane = t & 63;
            uint32_t a = 0;
            if (pat == kLaneBank && WIDTH == 2) {
                // 16-bit values in pairs: lane l's word at row * 256 + 4 * l, either half of it
                a = (uint32_t)(rnd() % (lds_bytes / 256)) * 256u + 4u * (uint32_t)lane + 2u * (rnd() & 1u);
            } else if (pat == kLaneBank) {
                const int rows = lds_bytes / (64 * WIDTH);
                a = (uint32_t)(rnd() % rows) * 64u * WIDTH + (uint32_t)lane * WIDTH;
            } else if (pat == kBroadcast) {
                a = (uint32_t)((u * 40 + (t >> 6) * 8) % (lds_bytes / WIDTH)) * WIDTH;
            } else if (pat == kRandomSmall) {
                a = (uint32_t)((t >> 6) * 2048 + u * 64) % (uint32_t)(lds_bytes - span) / 16 * 16 +
                    (uint32_t)(rnd() % (span / WIDTH)) * WIDTH;
            } else {
                a = (uint32_t)(rnd() % (lds_bytes / WIDTH)) * WIDTH;
            }
            h[(size_t)u * threads + t] = a;
        }
    uint32_t *d_addr;
    CK(hipMalloc(&d_addr, h.size() * 4));
    CK(hipMemcpy(d_addr, h.data(), h.size() * 4, hipMemcpyHostToDevice));
    auto kern = lds_read_kernel<WIDTH, U>;
    CK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    const int iters = 4000;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    kern<<<n_cu, threads, lds_bytes>>>(d_addr, lds_bytes, 10, d_out);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    kern<<<n_cu, threads, lds_bytes>>>(d_addr, lds_bytes, iters, d_out);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double reads_per_cu = (double)iters * U * waves;          // wavefront-wide reads
    const double clk = ms * 1e-3 * 2.4e9 / reads_per_cu;
    printf("  %-44s %2d waves: %6.2f clk per wavefront read per CU  (%6.1f B/clk/CU)\n", name, waves, clk,
           64.0 * WIDTH / clk);
    CK(hipFree(d_addr));
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return clk;
}

// Synthetic visit loop: K walks per lane in lock-step over `depth` levels of random perfect
// trees in the traversal kernel's node format (8 bytes: threshold, (feature*256)<<16 | left
// child offset, right child next to left), features in a lane-per-bank tile.
template <int K>
__global__ void __launch_bounds__(1024) visit_kernel(const uint32_t *__restrict__ image, int image_bytes, int n_trees,
                                                    int tree_bytes, int depth, int n_features, int rounds,
                                                    uint32_t *out)
{
    extern __shared__ uint32_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < image_bytes / 4; i += blockDim.x)
        lds[i] = image[i];
    const int tile0 = image_bytes;
    for (int i = tid; i < n_features * 64 * 2; i += blockDim.x)       // two tiles
        lds[tile0 / 4 + i] = __float_as_uint((float)((i * 2654435761u) >> 8) * (1.0f / 16777216.0f));
    __syncthreads();
    const uint32_t lane_base = (uint32_t)tile0 + (uint32_t)(wave & 1) * (uint32_t)n_features * 256u + 4u * (uint32_t)lane;
    uint32_t acc = 0;
    for (int r = 0; r < rounds; ++r) {
        uint32_t a[K];
#pragma unroll
        for (int k = 0; k < K; ++k)
            a[k] = (uint32_t)(((wave >> 1) * K + k + r) % n_trees) * (uint32_t)tree_bytes;
        for (int l = 0; l < depth; ++l) {
            u32x2 nd[K];
            float x[K];
#pragma unroll
            for (int k = 0; k < K; ++k)
                nd[k] = *(const u32x2 *)((const char *)lds + a[k]);
#pragma unroll
            for (int k = 0; k < K; ++k)
                x[k] = *(const float *)((const char *)lds + (nd[k].y >> 16) + lane_base);
#pragma unroll
            for (int k = 0; k < K; ++k)
                a[k] = (nd[k].y & 0xFFFFu) + ((x[k] < __uint_as_float(nd[k].x)) ? 0u : 8u);
        }
#pragma unroll
        for (int k = 0; k < K; ++k)
            acc ^= a[k];
    }
    if (acc == 0x12345678u)
        out[0] = acc;
}

static double run_visits(int waves, int depth, int n_cu, uint32_t *d_out)
{
    constexpr int K = 8;
    const int n_features = 164, lds_total = 160 * 1024;
    const int tree_nodes = (2 << depth) - 1, tree_bytes = ((tree_nodes * 8) + 15) & ~15;
    const int room = lds_total - 2 * n_features * 256 - 64;
    const int n_trees = room / tree_bytes;
    const int image_bytes = n_trees * tree_bytes;
    std::vector<uint32_t> img((size_t)image_bytes / 4, 0);
    for (int t = 0; t < n_trees; ++t)
        for (int n = 0; n < tree_nodes; ++n) {
            const uint32_t at = (uint32_t)(t * tree_bytes + n * 8);
            float thr = (float)(rnd() & 0xFFFF) / 65536.0f;
            uint32_t tb;
            __builtin_memcpy(&tb, &thr, 4);
            const bool leaf = 2 * n + 1 >= tree_nodes;
            const uint32_t child = leaf ? at - 8 + 0 : (uint32_t)(t * tree_bytes + (2 * n + 1) * 8);
            const uint32_t feat = leaf ? 0u : (uint32_t)(rnd() % n_features);
            img[at / 4] = tb;
            img[at / 4 + 1] = ((feat * 256u) << 16) | (child & 0xFFFFu);
        }
    uint32_t *d_img;
    CK(hipMalloc(&d_img, (size_t)image_bytes));
    CK(hipMemcpy(d_img, img.data(), (size_t)image_bytes, hipMemcpyHostToDevice));
    auto kern = visit_kernel<K>;
    CK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_total));
    const int rounds = 400;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    kern<<<n_cu, waves * 64, lds_total>>>(d_img, image_bytes, n_trees, tree_bytes, depth, n_features, 4, d_out);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    kern<<<n_cu, waves * 64, lds_total>>>(d_img, image_bytes, n_trees, tree_bytes, depth, n_features, rounds, d_out);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double visits_per_cu = (double)rounds * K * depth * waves;  // wavefront-wide visits
    const double clk = ms * 1e-3 * 2.4e9 / visits_per_cu;
    printf("  lock-step visit loop, depth %2d, %2d trees resident, %2d waves, K=%d: %6.2f clk per wavefront visit per CU"
           "  -> %.3e visits/s on %d CUs\n", depth, n_trees, waves, K, clk, 64.0 * n_cu * 2.4e9 / clk, n_cu);
    CK(hipFree(d_img));
    return clk;
}

// Synthetic walk over rank-coded data: 4-byte nodes in 1-based heap order without child
// pointers (rank << 16 | offset of the feature in a tile), 16-bit feature ranks in pairs, K walks
// per lane in lock-step -- the visit of the rank traversal kernel with nothing around it.
template <int K>
__global__ void __launch_bounds__(768) rank_visit_kernel(const uint32_t *__restrict__ image, int n_trees, int depth,
                                                         int n_features, int rounds, uint32_t *out)
{
    extern __shared__ uint32_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tree_words = 2 << depth, image_words = n_trees * tree_words;
    for (int i = tid; i < image_words; i += blockDim.x)
        lds[i] = image[i];
    const int tile0 = image_words * 4, cols = (n_features + 1) & ~1, tile_words = cols * 32;
    for (int i = tid; i < 4 * tile_words; i += blockDim.x)            // four tiles
        lds[tile0 / 4 + i] = (uint32_t)i * 2654435761u;
    __syncthreads();
    const uint32_t lane_base = (uint32_t)tile0 + (uint32_t)(wave & 3) * (uint32_t)tile_words * 4u + 4u * (uint32_t)lane;
    uint32_t acc = 0;
    for (int r = 0; r < rounds; ++r) {
        uint32_t base[K], A[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            base[k] = (uint32_t)(((wave >> 2) * K + k + r) % n_trees) * (uint32_t)tree_words * 4u;
            A[k] = base[k] + 4u;
        }
        for (int l = 0; l < depth; ++l) {
            uint32_t nd[K], x[K];
#pragma unroll
            for (int k = 0; k < K; ++k)
                nd[k] = *(const uint32_t *)((const char *)lds + A[k]);
#pragma unroll
            for (int k = 0; k < K; ++k)
                x[k] = *(const uint16_t *)((const char *)lds + (nd[k] & 0xFFFFu) + lane_base);
#pragma unroll
            for (int k = 0; k < K; ++k)
                A[k] = (A[k] << 1) - base[k] + ((x[k] < (nd[k] >> 16)) ? 0u : 4u);
        }
#pragma unroll
        for (int k = 0; k < K; ++k)
            acc ^= A[k];
    }
    if (acc == 0x12345678u)
        out[0] = acc;
}

template <int K>
static double run_rank_visits(int depth, int n_trees, int n_cu, uint32_t *d_out)
{
    const int n_features = 164, lds_total = 160 * 1024, waves = 12;
    const int tree_words = 2 << depth;
    std::vector<uint32_t> img((size_t)n_trees * tree_words, 0);
    for (int t = 0; t < n_trees; ++t)
        for (int i = 1; i < tree_words; ++i) {
            const uint32_t f = (uint32_t)(rnd() % n_features);
            img[(size_t)t * tree_words + i] = ((rnd() & 0xFFFFu) << 16) | ((f >> 1) * 256u + (f & 1u) * 2u);
        }
    uint32_t *d_img;
    CK(hipMalloc(&d_img, img.size() * 4));
    CK(hipMemcpy(d_img, img.data(), img.size() * 4, hipMemcpyHostToDevice));
    auto kern = rank_visit_kernel<K>;
    CK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_total));
    const int rounds = 400;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    kern<<<n_cu, waves * 64, lds_total>>>(d_img, n_trees, depth, n_features, 4, d_out);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    kern<<<n_cu, waves * 64, lds_total>>>(d_img, n_trees, depth, n_features, rounds, d_out);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double clk = ms * 1e-3 * 2.4e9 / ((double)rounds * K * depth * waves);
    printf("  rank walk, depth %2d, %2d trees resident, 12 waves, %d walks per lane (%3d in flight per CU): "
           "%6.2f clk per wavefront visit per CU -> %.3e visits/s\n", depth, n_trees, K, K * waves, clk,
           64.0 * n_cu * 2.4e9 / clk);
    CK(hipFree(d_img));
    return clk;
}

int main()
{
    hipDeviceProp_t p;
    CK(hipGetDeviceProperties(&p, 0));
    const int n_cu = p.multiProcessorCount;
    printf("device %s: %d CUs, %d kHz, LDS per workgroup %zu B\n", p.gcnArchName, n_cu, p.clockRate,
           p.sharedMemPerBlock);
    printf("(clocks below assume 2.4 GHz)\n");
    uint32_t *d_out;
    CK(hipMalloc(&d_out, 64));

    printf("HBM read stream\n");
    double best_gbs = 0.0;
    for (size_t mb : {1400, 4300}) {
        const size_t bytes = mb << 20;
        u32x4 *d;
        CK(hipMalloc(&d, bytes));
        CK(hipMemset(d, 1, bytes));
        hipEvent_t e0, e1;
        CK(hipEventCreate(&e0));
        CK(hipEventCreate(&e1));
        for (int unroll : {1, 4})
            for (int blocks : {n_cu * 8, n_cu * 16, n_cu * 32}) {
                auto kern = unroll == 1 ? stream_read_kernel<1> : stream_read_kernel<4>;
                kern<<<blocks, 512>>>(d, bytes / 16, d_out);
                CK(hipDeviceSynchronize());
                CK(hipEventRecord(e0));
                for (int r = 0; r < 5; ++r)
                    kern<<<blocks, 512>>>(d, bytes / 16, d_out);
                CK(hipEventRecord(e1));
                CK(hipEventSynchronize(e1));
                float ms;
                CK(hipEventElapsedTime(&ms, e0, e1));
                ms /= 5;
                const double gbs = bytes / (ms * 1e-3) / 1e9;
                printf("  %5zu MiB, %5d workgroups of 512, %d load(s) in flight per thread: %.3f ms = %.0f GB/s\n",
                       mb, blocks, unroll, ms, gbs);
                if (gbs > best_gbs)
                    best_gbs = gbs;
            }
        CK(hipFree(d));
    }

    printf("LDS reads, independent loads (8 per lane and iteration), 64 KB buffer\n");
    double b32_cf = 1e9, b64_cf = 1e9, b64_small = 1e9, b64_all = 1e9, b64_bc = 1e9;
    for (int waves : {8, 12, 16}) {
        double c;
        c = run_lds<4, 8>("b32, lane in its own bank (a feature read)", kLaneBank, waves, 65536, 0, n_cu, d_out);
        if (c < b32_cf) b32_cf = c;
        c = run_lds<8, 8>("b64, lane in its own banks (conflict-free)", kLaneBank, waves, 65536, 0, n_cu, d_out);
        if (c < b64_cf) b64_cf = c;
        c = run_lds<8, 8>("b64, all lanes one address (a root)", kBroadcast, waves, 65536, 0, n_cu, d_out);
        if (c < b64_bc) b64_bc = c;
        c = run_lds<8, 8>("b64, random within 128 B (level 4, 16 nodes)", kRandomSmall, waves, 65536, 128, n_cu, d_out);
        c = run_lds<8, 8>("b64, random within 1 KB (level 7, 128 nodes)", kRandomSmall, waves, 65536, 1024, n_cu, d_out);
        if (c < b64_small) b64_small = c;
        c = run_lds<8, 8>("b64, random over 64 KB", kRandomAll, waves, 65536, 0, n_cu, d_out);
        if (c < b64_all) b64_all = c;
        run_lds<16, 8>("b128, lane in its own banks", kLaneBank, waves, 65536, 0, n_cu, d_out);
        if (waves == 12) {
            run_lds<2, 8>("u16, lane in its own bank (a rank-coded feature)", kLaneBank, waves, 65536, 0, n_cu, d_out);
            run_lds<4, 8>("b32, random within 256 B (64 4-byte nodes)", kRandomSmall, waves, 65536, 256, n_cu, d_out);
            run_lds<4, 8>("b32, random within 1 KB (256 4-byte nodes)", kRandomSmall, waves, 65536, 1024, n_cu, d_out);
            run_lds<4, 8>("b32, random within 4 KB (1024 4-byte nodes)", kRandomSmall, waves, 65536, 4096, n_cu, d_out);
            run_lds<16, 8>("b128, random within 1 KB (64 16-byte nodes)", kRandomSmall, waves, 65536, 1024, n_cu, d_out);
            run_lds<16, 8>("b128, random within 4 KB (256 16-byte nodes)", kRandomSmall, waves, 65536, 4096, n_cu, d_out);
        }
    }

    printf("Synthetic lock-step visit loop (8-byte nodes, fp32 tile, two tiles, whole LDS)\n");
    double visit8 = 1e9, visit6 = 1e9;
    for (int waves : {8, 12, 16}) {
        double c = run_visits(waves, 8, n_cu, d_out);
        if (c < visit8) visit8 = c;
        c = run_visits(waves, 6, n_cu, d_out);
        if (c < visit6) visit6 = c;
    }
    printf("Synthetic walk over rank-coded data (4-byte heap nodes, 16-bit feature ranks, four tiles)\n");
    run_rank_visits<2>(10, 8, n_cu, d_out);
    const double rank3 = run_rank_visits<3>(10, 8, n_cu, d_out);
    run_rank_visits<4>(10, 8, n_cu, d_out);
    run_rank_visits<5>(10, 8, n_cu, d_out);
    const double rank8 = run_rank_visits<8>(10, 8, n_cu, d_out);
    run_rank_visits<8>(8, 32, n_cu, d_out);
    const double visit_peak = 64.0 * n_cu * 2.4e9 / (b64_cf + b32_cf);
    printf("JSON {\"hbm_read_stream_gbs\": %.0f, \"lds_b32_lane_bank_clk\": %.3f, \"lds_b64_lane_bank_clk\": %.3f, "
           "\"lds_b64_broadcast_clk\": %.3f, \"lds_b64_random_1k_clk\": %.3f, \"lds_b64_random_64k_clk\": %.3f, "
           "\"visit_loop_depth8_clk\": %.3f, \"visit_loop_depth6_clk\": %.3f, \"visit_peak_conflict_free\": %.4e, "
           "\"visit_loop_measured\": %.4e, \"rank_walk_depth10_k3_clk\": %.3f, \"rank_walk_depth10_k8_clk\": %.3f, "
           "\"cus\": %d}\n",
           best_gbs, b32_cf, b64_cf, b64_bc, b64_small, b64_all, visit8, visit6, visit_peak,
           64.0 * n_cu * 2.4e9 / visit8, rank3, rank8, n_cu);
    CK(hipFree(d_out));
    return 0;
}
