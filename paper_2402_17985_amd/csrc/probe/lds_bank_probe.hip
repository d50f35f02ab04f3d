// LDS bank-conflict probe for gfx950 (a measurement tool, not part of libfq.so).
//
// One workgroup of 8 waves reads LDS in a loop; every wave uses the same per-lane address table.  The
// figure printed is core-clock cycles per wave-level read instruction at saturation, for 16-byte
// (ds_read_b128) and 8-byte (ds_read_b64) reads: the conflict-free value is the LDS's rate, multiples of
// it are bank conflicts.  The tables probe (i) the bank geometry (strides), (ii) which lanes share a pass
// (lane l and lane l | k made to collide), and (iii) the operand-read patterns of the 6-bit GEMM for the
// family of layouts "swap the two 48-byte groups of a 96-byte row where parity(row & sw) is odd; take the
// mirrored unit where parity(row & mr) ^ k-half is odd", printing the pairs (sw, mr) for which both reads
// run at the conflict-free rate.
//
// Build and run (on an MI355X):
//   hipcc --offload-arch=gfx950 -O3 -o lds_bank_probe paper_2402_17985_amd/csrc/probe/lds_bank_probe.hip
//   ./lds_bank_probe
#include <hip/hip_runtime.h>
#include <cstdio>
#include <string>
#include <vector>
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            printf("%s failed: %s\n", #x, hipGetErrorString(e_));                     \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

template <int W>
__global__ void probe(const int* __restrict__ addr, int iters, long long* out, int* sink)
{
    extern __shared__ __align__(16) unsigned char lds[];
    for (int i = threadIdx.x; i < 16384; i += blockDim.x) reinterpret_cast<int*>(lds)[i] = i;
    __syncthreads();
    const int a = addr[threadIdx.x & 63];          // checked on the host: a + W <= 65536, a % W == 0
    int acc = 0;
    const long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
        if (W == 16) {
            v4i v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) asm volatile("ds_read_b128 %0, %1" : "=v"(v[u]) : "v"(a));
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u][0];
        } else {
            v2i v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) asm volatile("ds_read_b64 %0, %1" : "=v"(v[u]) : "v"(a));
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u][0];
        }
    }
    __syncthreads();
    const long long t1 = __builtin_readcyclecounter();
    if (threadIdx.x == 0) out[0] = t1 - t0;
    sink[threadIdx.x & 63] = acc;
}

int main()
{
    int *d_addr, *d_sink;
    long long* d_out;
    CHECK(hipMalloc(&d_addr, 64 * 4));
    CHECK(hipMalloc(&d_sink, 64 * 4));
    CHECK(hipMalloc(&d_out, 8));
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(probe<16>), hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(probe<8>), hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
    // cycles per wave-read of an address table, or -1 if the table leaves the 64 KiB window
    auto measure = [&](int W, const std::vector<int>& a, int iters) -> double {
        for (int x : a)
            if (x < 0 || x + W > 65536 || x % W) return -1.0;
        if (hipMemcpy(d_addr, a.data(), 64 * 4, hipMemcpyHostToDevice) != hipSuccess) return -1.0;
        long long c = 0;
        for (int rep = 0; rep < 2; ++rep) {
            if (W == 16) probe<16><<<1, 512, 65536>>>(d_addr, iters, d_out, d_sink);
            else probe<8><<<1, 512, 65536>>>(d_addr, iters, d_out, d_sink);
            if (hipDeviceSynchronize() != hipSuccess) return -1.0;
            if (hipMemcpy(&c, d_out, 8, hipMemcpyDeviceToHost) != hipSuccess) return -1.0;
        }
        return (double)c / (iters * 8.0 * 8.0);
    };
    auto run = [&](const char* name, int W, const std::vector<int>& a) {
        printf("%-46s %2d-byte reads  %6.2f cycles per wave-read\n", name, W, measure(W, a, 2000));
        fflush(stdout);
    };
    for (int W : {16, 8}) {
        std::vector<int> a(64);
        for (int l = 0; l < 64; ++l) a[l] = W * l;
        run("consecutive lanes, consecutive addresses", W, a);
        for (int l = 0; l < 64; ++l) a[l] = 0;
        run("all lanes one address", W, a);
        for (int stride : {128, 256, 512}) {
            for (int l = 0; l < 64; ++l) a[l] = stride * l;
            run(("lane stride " + std::to_string(stride) + " bytes").c_str(), W, a);
        }
        // lanes l and l | k sit on the same banks, 4096 bytes apart (+128: half a bank cycle further)
        for (int shift : {0, 128})
            for (int k : {1, 2, 4, 8, 16, 32}) {
                for (int l = 0; l < 64; ++l) a[l] = W * (l & ~k) + ((l & k) ? 4096 + shift : 0);
                run(("lanes l, l|" + std::to_string(k) + " collide, partner at +4096" + (shift ? "+128" : "")).c_str(), W, a);
            }
    }
    // operand reads of the 6-bit GEMM: LDS rows of 96 bytes; lane = (row l % 32, k-half l / 32)
    auto par = [](int v) { return __builtin_popcount(v) & 1; };
    auto tables = [&](int sw, int mr, std::vector<int>& x, std::vector<int>& y) {
        for (int l = 0; l < 64; ++l) {
            const int row = l & 31, h = l >> 5;
            const int m = h ^ par(row & mr);
            x[l] = row * 96 + 48 * par(row & sw) + (m ? 32 : 0);
            y[l] = row * 96 + 48 * par(row & sw) + (m ? 24 : 16);
        }
    };
    std::vector<int> x(64), y(64);
    struct { int sw, mr; const char* what; } named[] = {
        {8, 0, "swap on row bit 3, unit by k-half"},
        {8, 16, "swap on row bit 3, unit mirrored on row bit 4"},
        {12, 16, "swap on row bits 2^3, mirrored on bit 4 (used)"},
    };
    for (auto& n : named) {
        tables(n.sw, n.mr, x, y);
        run((std::string("GEMM 16-byte piece: ") + n.what).c_str(), 16, x);
        run((std::string("GEMM  8-byte piece: ") + n.what).c_str(), 8, y);
    }
    int good = 0;
    printf("layouts (sw, mr) with both reads conflict free:");
    for (int sw = 0; sw < 32; ++sw)
        for (int mr = 0; mr < 32; ++mr) {
            tables(sw, mr, x, y);
            const double cx = measure(16, x, 300), cy = measure(8, y, 300);
            if (cx > 0 && cx < 4.5 && cy > 0 && cy < 3.0) {
                printf(" (%d,%d)", sw, mr);
                ++good;
            }
        }
    printf("\n%d of 1024 layouts\n", good);
    return 0;
}
