// LDS bank structure probe for gfx950 (diagnostic, not part of the library).
//
// Times ds_read_b128 / ds_read_b32 issued back to back by every wave of one workgroup per CU, for a set of
// per-lane address patterns, and prints the cost per wave-instruction as seen by the CU.  It is what the
// LDS layouts of the skinny GEMM's table kernel (staged X, sign table copies) are derived from:
//   * a conflict-free ds_read_b128 costs about 4 clocks per wave (256 B/clk per CU) with 16 waves per CU;
//   * it is served 16 lanes at a time in the groups {0-3, 12-15, 20-23, 24-27}, {4-7, 8-11, 16-19, 28-31}
//     and the same plus 32, and a group is conflict-free when its 16 addresses fall into 16 different
//     16-byte columns of a 256-byte row (64 banks of 4 bytes), or are equal;
//   * a ds_read_b32 is conflict-free over 64 consecutive dwords (about 2 clocks per wave).
// The model is printed next to each measurement ("passes" = sum over the groups of the largest number of
// different addresses that share a 16-byte column; 4 = conflict-free).
//
// Build and run:  python -m paper_2407_02891_amd.build --probes && paper_2407_02891_amd/probes/lds_banks
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <set>
#include <string>
#include <vector>

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr int K = 16;              // reads in flight per wave and iteration
constexpr int kLdsBytes = 96 * 1024;

template <int WIDE>
__global__ __launch_bounds__(1024) void probe(const int *addr, unsigned long long *out, int iters)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[kLdsBytes];
    const int lane = threadIdx.x & 63;
    for (int i = threadIdx.x; i < kLdsBytes / 4; i += blockDim.x) reinterpret_cast<unsigned *>(lds)[i] = i * 2654435761u;
    int a[K];
#pragma unroll
    for (int k = 0; k < K; ++k) a[k] = addr[k * 64 + lane];
    const unsigned base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds;
#pragma unroll
    for (int k = 0; k < K; ++k) a[k] += base;
    unsigned acc = 0;
    __syncthreads();
    const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
        if (WIDE) {
            u32x4 v[K];
#pragma unroll
            for (int k = 0; k < K; ++k) asm volatile("ds_read_b128 %0, %1" : "=v"(v[k]) : "v"(a[k]));
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]));
            asm volatile("" : "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15]));
#pragma unroll
            for (int k = 0; k < K; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
        } else {
            unsigned v[K];
#pragma unroll
            for (int k = 0; k < K; ++k) asm volatile("ds_read_b32 %0, %1" : "=v"(v[k]) : "v"(a[k]));
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]));
            asm volatile("" : "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15]));
#pragma unroll
            for (int k = 0; k < K; ++k) acc ^= v[k];
        }
    }
    const unsigned long long t1 = __builtin_amdgcn_s_memrealtime();  // 100 MHz
    if (lane == 0) out[blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6)] = t1 - t0;
    if (acc == 0x12345u) out[8000] = acc;  // keeps the reads alive
}

static unsigned g_rng = 12345;
static unsigned rnd()
{
    g_rng = g_rng * 1664525u + 1013904223u;
    return g_rng >> 8;
}

struct Pattern {
    std::string name;
    int wide;
    std::vector<int> a;  // [K][64] byte addresses
};

// The model: passes of a ds_read_b128 over its four lane groups.
static double model_passes(const Pattern &p)
{
    static const int first[2][4] = {{0, 12, 20, 24}, {4, 8, 16, 28}};
    double total = 0;
    for (int k = 0; k < K; ++k)
        for (int half = 0; half < 2; ++half)
            for (int g = 0; g < 2; ++g) {
                std::set<int> column[16];
                for (int q = 0; q < 4; ++q)
                    for (int j = 0; j < 4; ++j) {
                        const int lane = 32 * half + first[g][q] + j, addr = p.a[k * 64 + lane];
                        column[(addr >> 4) & 15].insert(addr);
                    }
                size_t worst = 0;
                for (auto &c : column) worst = c.size() > worst ? c.size() : worst;
                total += (double)worst;
            }
    return total / K;
}

#define CHECK(x)                                                             \
    do {                                                                     \
        hipError_t e_ = (x);                                                 \
        if (e_ != hipSuccess) {                                              \
            printf("%s failed: %s\n", #x, hipGetErrorString(e_));           \
            return 1;                                                        \
        }                                                                    \
    } while (0)

int main()
{
    int *d_addr;
    unsigned long long *d_out;
    CHECK(hipMalloc(&d_addr, K * 64 * sizeof(int)));
    CHECK(hipMalloc(&d_out, 8192 * sizeof(unsigned long long)));
    std::vector<Pattern> pats;
    auto add = [&](const char *name, int wide, auto f) {
        Pattern p;
        p.name = name;
        p.wide = wide;
        p.a.resize(K * 64);
        for (int k = 0; k < K; ++k)
            for (int l = 0; l < 64; ++l) {
                const int v = f(k, l);
                if (v < 0 || v + 16 > kLdsBytes || (v & (wide ? 15 : 3))) {  // every access stays inside the array
                    printf("bad address %d in %s\n", v, name);
                    exit(1);
                }
                p.a[k * 64 + l] = v;
            }
        pats.push_back(p);
    };
    add("b128 lane*16 (linear)", 1, [](int k, int l) { return l * 16 + k * 1024; });
    add("b128 one address for all lanes", 1, [](int k, int) { return k * 1024; });
    add("b128 stride 32 B", 1, [](int k, int l) { return l * 32 + k * 2048; });
    add("b128 stride 64 B", 1, [](int k, int l) { return l * 64 + k * 4096; });
    add("b128 stride 128 B", 1, [](int k, int l) { return l * 128 + k * 16; });
    add("b128 stride 256 B", 1, [](int k, int l) { return l * 256 + k * 16; });
    add("b128 sign table, 16 copies (lane&15), random byte", 1, [](int, int l) { return (int)((rnd() & 255) * 16 + (l & 15)) * 16; });
    add("b128 sign table, 8 copies (lane&7), random byte", 1, [](int, int l) { return (int)((rnd() & 255) * 8 + (l & 7)) * 16; });
    add("b128 sign table, 8 copies, same byte in all lanes", 1, [](int k, int l) { return (int)((k * 37 & 255) * 8 + (l & 7)) * 16; });
    add("b128 sign table, 1 copy, random byte", 1, [](int, int) { return (int)(rnd() & 255) * 16; });
    add("b128 X r*1040 + h*64 + k*16 (chunk order 4h+s)", 1, [](int k, int l) { return (l & 15) * 1040 + (l >> 4) * 64 + k * 16; });
    add("b128 X r*1056 + h*16 + k*64 (chunk order 4s+h)", 1, [](int k, int l) { return (l & 15) * 1056 + (l >> 4) * 16 + k * 64; });
    add("b128 X r*1040 + h*256 + k*16 (one block per h)", 1, [](int k, int l) { return (l & 15) * 1040 + (l >> 4) * 256 + k * 16; });
    add("b128 X r*1024 + h*64 + k*16 (no padding)", 1, [](int k, int l) { return (l & 15) * 1024 + (l >> 4) * 64 + k * 16; });
    add("b32 lane*4 (linear)", 0, [](int k, int l) { return l * 4 + k * 256; });
    add("b32 stride 8 B", 0, [](int k, int l) { return l * 8 + k * 512; });
    add("b32 stride 256 B", 0, [](int k, int l) { return l * 256 + k * 4; });
    add("b32 GEMV table: (random index)*256 + lane*4", 0, [](int, int l) { return (int)(rnd() & 255) * 256 + l * 4; });
    const int iters = 2000;
    for (int waves : {8, 16}) {
        printf("--- %d waves per workgroup, one workgroup per CU (256 workgroups); clocks assume 2.4 GHz ---\n", waves);
        for (auto &p : pats) {
            CHECK(hipMemcpy(d_addr, p.a.data(), K * 64 * sizeof(int), hipMemcpyHostToDevice));
            double best = 1e30;
            for (int rep = 0; rep < 3; ++rep) {
                if (p.wide) hipLaunchKernelGGL(probe<1>, dim3(256), dim3(64 * waves), 0, 0, d_addr, d_out, iters);
                else hipLaunchKernelGGL(probe<0>, dim3(256), dim3(64 * waves), 0, 0, d_addr, d_out, iters);
                CHECK(hipGetLastError());
                CHECK(hipDeviceSynchronize());
                std::vector<unsigned long long> o(256 * waves);
                CHECK(hipMemcpy(o.data(), d_out, o.size() * sizeof(o[0]), hipMemcpyDeviceToHost));
                double s = 0;
                for (auto v : o) s += (double)v;
                s /= (double)o.size();
                best = s < best ? s : best;
            }
            const double ns = best * 10.0 / ((double)iters * K * waves);  // per wave-instruction, as seen by the CU
            if (p.wide)
                printf("%-52s %6.2f clk per wave-instruction, %6.1f B/clk per CU; model: %5.2f passes\n", p.name.c_str(),
                       ns * 2.4, 1024.0 / (ns * 2.4), model_passes(p));
            else
                printf("%-52s %6.2f clk per wave-instruction, %6.1f B/clk per CU\n", p.name.c_str(), ns * 2.4, 256.0 / (ns * 2.4));
            fflush(stdout);
        }
    }
    return 0;
}
