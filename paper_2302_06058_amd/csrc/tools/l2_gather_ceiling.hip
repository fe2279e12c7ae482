// Measurement tool (not part of libbimask.so): how fast can the CUs of a gfx950 pull 128-byte rows of an
// L2-resident bit matrix through a row permutation?  That is the access pattern of the permutation
// search of Sec. 3.3 / Alg. 1 (arXiv 2302.06058): for each of K candidates P_c every mask row is read once
// through P_c, K * I * J / 8 bytes in total, while the matrix itself (I * J / 8 bytes) stays in L2.
//
// The kernel below issues exactly the loads of the library's scoring kernel for the 2:4 case -- a
// wavefront = (column slice of 1024 columns = 128 bytes per row, candidate, range of row blocks); lane
// (b, q) = (lane / 8, lane % 8) reads the 16-byte piece q of the 4 rows of row block b through the
// candidate; two row-block groups (16 blocks) in flight per step; slices handed to the XCDs as
// contiguous runs -- and replaces the counting arithmetic by one XOR per loaded word.  Its rate is the
// ceiling the scoring kernel can be measured against.  A second figure reads the same slice
// rows in order (no permutation) for comparison.
//
//   build:  hipcc --offload-arch=gfx950 -O3 -o l2_gather_ceiling l2_gather_ceiling.hip
//   run:    ./l2_gather_ceiling            (prints one line per shape)
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); std::exit(1); } } while (0)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(256)
k_gather(const uint32_t* __restrict__ bits, int I, int wpr32, const int32_t* __restrict__ perms, int K, int nseg, int sps,
         int64_t items, uint32_t* __restrict__ sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t per_xcd = gridDim.x / 8;
    const int64_t item = ((blockIdx.x % 8) * per_xcd + blockIdx.x / 8) * 4 + wave;
    if (item >= items) return;
    const int seg = static_cast<int>(item % nseg);
    const int64_t sc = item / nseg;
    const int c = static_cast<int>(sc % K), slice = static_cast<int>(sc / K);
    const int bl = lane >> 3, ch = lane & 7;
    const uint32_t* Bs = bits + (slice * 8 + ch) * 4;
    const int nblk = I / 4, steps = (nblk + 15) / 16;
    const int s_begin = seg * sps, s_end = s_begin + sps < steps ? s_begin + sps : steps;
    const int32_t* P = perms ? perms + static_cast<int64_t>(c) * I : nullptr;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int s = s_begin; s < s_end; ++s) {
        u32x4 x[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            int b = (s * 2 + u) * 8 + bl;
            b = b < nblk ? b : nblk - 1;
            int4 pe = P ? *reinterpret_cast<const int4*>(P + b * 4) : make_int4(4 * b, 4 * b + 1, 4 * b + 2, 4 * b + 3);
            x[u][0] = *reinterpret_cast<const u32x4*>(Bs + static_cast<int64_t>(pe.x) * wpr32);
            x[u][1] = *reinterpret_cast<const u32x4*>(Bs + static_cast<int64_t>(pe.y) * wpr32);
            x[u][2] = *reinterpret_cast<const u32x4*>(Bs + static_cast<int64_t>(pe.z) * wpr32);
            x[u][3] = *reinterpret_cast<const u32x4*>(Bs + static_cast<int64_t>(pe.w) * wpr32);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int m = 0; m < 4; ++m) acc ^= x[u][m];
    }
    const uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x9E3779B9u) sink[0] = r;                   // never true in practice: keeps the loads alive
}

static void measure(int I, int J, int K) {
    const int wpr32 = J / 32, nslices = J / 1024;
    const int nblk = I / 4, steps = (nblk + 15) / 16;
    int64_t nseg = (8192 + static_cast<int64_t>(nslices) * K - 1) / (static_cast<int64_t>(nslices) * K);
    const int64_t nseg_max = steps / 2 > 1 ? steps / 2 : 1;
    nseg = nseg < 1 ? 1 : (nseg > nseg_max ? nseg_max : nseg);
    const int sps = static_cast<int>((steps + nseg - 1) / nseg);
    nseg = (steps + sps - 1) / sps;
    const int64_t items = static_cast<int64_t>(nslices) * nseg * K;
    const unsigned grid = static_cast<unsigned>(((items + 3) / 4 + 7) / 8 * 8);
    std::mt19937 rng(12345);
    std::vector<uint32_t> hb(static_cast<size_t>(I) * wpr32);
    for (auto& w : hb) w = rng();
    std::vector<int32_t> hp(static_cast<size_t>(K) * I);
    for (int c = 0; c < K; ++c) {
        int32_t* p = hp.data() + static_cast<size_t>(c) * I;
        for (int i = 0; i < I; ++i) p[i] = i;
        for (int i = I - 1; i > 0; --i) std::swap(p[i], p[rng() % (i + 1)]);
    }
    uint32_t *db, *sink; int32_t* dp;
    CHECK(hipMalloc(&db, hb.size() * 4)); CHECK(hipMalloc(&dp, hp.size() * 4)); CHECK(hipMalloc(&sink, 64));
    CHECK(hipMemcpy(db, hb.data(), hb.size() * 4, hipMemcpyHostToDevice));
    CHECK(hipMemcpy(dp, hp.data(), hp.size() * 4, hipMemcpyHostToDevice));
    hipEvent_t a, b; CHECK(hipEventCreate(&a)); CHECK(hipEventCreate(&b));
    double us[2];
    for (int mode = 0; mode < 2; ++mode) {
        const int32_t* P = mode == 0 ? dp : nullptr;
        for (int w = 0; w < 5; ++w) hipLaunchKernelGGL(k_gather, dim3(grid), dim3(256), 0, 0, db, I, wpr32, P, K, (int)nseg, sps, items, sink);
        const int reps = 20;
        CHECK(hipEventRecord(a));
        for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(k_gather, dim3(grid), dim3(256), 0, 0, db, I, wpr32, P, K, (int)nseg, sps, items, sink);
        CHECK(hipEventRecord(b)); CHECK(hipEventSynchronize(b));
        float ms; CHECK(hipEventElapsedTime(&ms, a, b));
        us[mode] = ms * 1e3 / reps;
    }
    const double bytes = static_cast<double>(K) * I * J / 8;
    std::printf("I=%d J=%d K=%d: mask %.2f MB, gathered %.1f MB per search; through the permutations %.1f us = %.2f TB/s; "
                "rows in order %.1f us = %.2f TB/s\n", I, J, K, I * (J / 8.0) / 1e6, bytes / 1e6, us[0], bytes / us[0] / 1e6,
                us[1], bytes / us[1] / 1e6);
    CHECK(hipFree(db)); CHECK(hipFree(dp)); CHECK(hipFree(sink));
}

int main() {
    measure(11008, 4096, 100);     // W_up of the MLP block
    measure(4096, 11264, 100);     // W_down, columns rounded to whole 1024-column slices
    measure(256, 2048, 100);       // the ResNet-50 layer3 3x3 convolution, columns rounded down to whole slices
    measure(1024, 1024, 100);
    return 0;
}
