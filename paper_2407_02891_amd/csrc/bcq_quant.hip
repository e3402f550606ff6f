// The GPTQT quantiser for one linear layer with row-wise parameters (paper Sec. II-A Eq. 1-2,
// Sec. II-B Eq. 5-6, Sec. II-C Eq. 7 and the algorithm that closes Sec. II-D), the step that
// produces what bcq_from_linear_rows / bcq_pack consume.  Offline tooling: written for clarity
// and determinism (fixed reduction orders), not tuned.
//
//   search   per row m: qbias = min w, range = max w - min w; for S' on `grid` equidistant points
//            inside (range / (2^(n+1) - 1), range / (2^(n-1) - 1))  (Eq. 7), for every way of tying
//            the n linear bit-planes into q classes (Eq. 10): W_q = nearest member of that tying's
//            BCchoice to clamp(rne((w - qbias) / S'))  (Eq. 5 step 1, Eq. 6), output error
//            e = d (H / 2) d^T with d = S' W_q + qbias - w  (Eq. 5 step 2); the first candidate
//            with the smallest error is kept (scale-major order).
//   gptq     column by column, quant(w) = S W_q + qbias with the row's parameters; the error of
//            column j, divided by U[j][j], is spread over the later columns along row j of U, the
//            upper Cholesky factor of H^-1 (Eq. 2 in its usual one-factorisation form).
//
// The integer decisions (rounding to the linear grid, nearest BCchoice) are taken in binary64 from
// binary64 copies of the binary32 inputs; the quadratic form and the GPTQ updates run in binary32.
#include <algorithm>
#include <vector>

#include "bcq_internal.h"
#include "bcq_device.h"
#include "bcq_tying.h"

namespace bcq {

// One way of tying the planes: class of every bit, and the integers it can represent (ascending).
struct Tying {
    int8_t label[kMaxBits];
    int nchoice;
    int choice[16];
};

// All partitions of the planes 1..n into q non-empty classes; classes ordered by their smallest
// plane, partitions ordered lexicographically by their classes (shorter class first on a tie of
// the common prefix).
static std::vector<Tying> all_tyings(int n, int q)
{
    std::vector<std::vector<std::vector<int>>> parts;
    std::vector<int> lab(n, 0);
    // restricted growth strings: lab[0] = 0, lab[i] <= 1 + max(lab[0..i-1])
    std::vector<int> stack;
    struct Rec {
        static void go(int i, int n, int q, int used, std::vector<int> &lab,
                       std::vector<std::vector<std::vector<int>>> &out)
        {
            if (i == n) {
                if (used != q) return;
                std::vector<std::vector<int>> p(q);
                for (int k = 0; k < n; ++k) p[lab[k]].push_back(k + 1);
                out.push_back(p);
                return;
            }
            for (int c = 0; c <= used && c < q; ++c) {
                lab[i] = c;
                go(i + 1, n, q, c == used ? used + 1 : used, lab, out);
            }
        }
    };
    Rec::go(0, n, q, 0, lab, parts);
    std::sort(parts.begin(), parts.end());
    std::vector<Tying> out;
    for (const auto &p : parts) {
        Tying t{};
        for (int c = 0; c < q; ++c)
            for (int plane : p[c]) t.label[plane - 1] = (int8_t)c;
        TyingPlan plan;
        make_tying_plan(n, q, t.label, false, &plan);
        t.nchoice = plan.nchoice;
        std::copy(plan.choice, plan.choice + plan.nchoice, t.choice);
        out.push_back(t);
    }
    return out;
}

// Eq. 5 step 1 and Eq. 6 for one weight, in binary64.
__device__ __forceinline__ int quant_int(double w, double S, double qbias, int n_bits, const int *choice, int nchoice)
{
    double v = rint((w - qbias) / S);  // round half to even
    const double top = (double)((1 << n_bits) - 1);
    v = v < 0.0 ? 0.0 : (v > top ? top : v);
    return nearest_choice((int)v, choice, nchoice);
}

// ---------------------------------------------------------------------------------
// working layout
// ---------------------------------------------------------------------------------
// Both steps work on transposed binary32 copies, [column k][row m] with the row index fastest and a
// pitch Mp = M rounded up to 4: one thread per row then reads and writes coalesced, and both dense
// products below take their operands "k-major" (a tile is 16 values of the summation index by 128
// contiguous floats).  Workspace, in floats:
//   Wt [N][Mp] | Dt [N][Mp] | part [ceil(N/128)][Mp] | wmin, wmax, best [3][Mp] | Err [128][Mp]
struct QuantWorkspace {
    int Mp, ntile;
    float *Wt, *Dt, *part, *wmin, *wmax, *best, *Err;
};

static int pitch_of(int M) { return (M + 3) / 4 * 4; }

static QuantWorkspace carve(void *workspace, int M, int N)
{
    QuantWorkspace w;
    w.Mp = pitch_of(M);
    w.ntile = (N + 127) / 128;
    w.Wt = static_cast<float *>(workspace);
    w.Dt = w.Wt + (size_t)N * w.Mp;
    w.part = w.Dt + (size_t)N * w.Mp;
    w.wmin = w.part + (size_t)w.ntile * w.Mp;
    w.wmax = w.wmin + w.Mp;
    w.best = w.wmax + w.Mp;
    w.Err = w.best + w.Mp;
    return w;
}

size_t quant_workspace_bytes(int M, int N)
{
    const size_t Mp = pitch_of(M), ntile = (size_t)(N + 127) / 128;
    const size_t floats = 2 * (size_t)N * Mp + ntile * Mp + 3 * Mp + 128 * Mp;
    return (floats * 4 + 255) / 256 * 256;
}

// Wt[k][m] = W[m][k]; the pad rows m in [M, Mp) are written as zeros.
__global__ void transpose_kernel(int M, int Mp, int N, const float *__restrict__ W, float *__restrict__ Wt)
{
    __shared__ float tile[32][33];
    const int m0 = blockIdx.y * 32, k0 = blockIdx.x * 32;
    for (int i = threadIdx.y; i < 32; i += blockDim.y) {
        const int m = m0 + i, k = k0 + threadIdx.x;
        tile[i][threadIdx.x] = (m < M && k < N) ? W[(size_t)m * N + k] : 0.0f;
    }
    __syncthreads();
    for (int i = threadIdx.y; i < 32; i += blockDim.y) {
        const int k = k0 + i, m = m0 + threadIdx.x;
        if (m < Mp && k < N) Wt[(size_t)k * Mp + m] = tile[threadIdx.x][i];
    }
}

// ---------------------------------------------------------------------------------
// dense product on the matrix cores, binary32:  C[r][c] = sum_k A[k][r] * B[k][c]
// ---------------------------------------------------------------------------------
// A is [K][R] with pitch lda, B is [K][C] with pitch ldb (both pitches and R, C multiples of 4, all
// pointers 16-byte aligned).  A workgroup of four waves owns a 128 x 128 tile of C, a wave a 64 x 64
// quarter as 2 x 2 v_mfma_f32_32x32x2_f32 accumulators; the operand tiles (16 k x 128) go through
// LDS, double-buffered, the next pair of tiles travelling through registers while the current one
// is multiplied.  What happens to the finished tile is the caller's epilogue:
//   kQuadForm   part[tile row][c] = sum over the tile's rows r of C[r][c] * E[r][c]; A symmetric, E = B
//               (the k range stops at the tile's last row, see the loader)
//   kSubtract   Out[r][c] -= C[r][c]
//   kAddTwice   Out[r][c] += 2 C[r][c]
//   kStore      Out[r][c] = C[r][c];   kStoreNegated   Out[r][c] = -C[r][c]
// (Out and E have pitch ldo; for kQuadForm Out is [tile row][ldo].)
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4v __attribute__((ext_vector_type(4)));
enum { kQuadForm = 0, kSubtract = 1, kAddTwice = 2, kStore = 3, kStoreNegated = 4 };
constexpr int kTile = 128, kStep = 16;

__device__ __forceinline__ f32x4v load4_or_zero(const float *base, size_t pitch, int k, int K, int x, int X)
{
    if (k < K && x < X) return *reinterpret_cast<const f32x4v *>(base + (size_t)k * pitch + x);
    return f32x4v{0.f, 0.f, 0.f, 0.f};
}

template <int MODE>
__global__ __launch_bounds__(256) void mfma_kmajor_kernel(const float *__restrict__ A, int lda, int R,
                                                          const float *__restrict__ B, int ldb, int C, int K,
                                                          float *__restrict__ out, int ldo, const float *__restrict__ E)
{
    __shared__ __attribute__((aligned(16))) float As[2][kStep][kTile];
    __shared__ __attribute__((aligned(16))) float Bs[2][kStep][kTile];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lo = lane & 31, hi = lane >> 5;
    const int wr = wave >> 1, wc = wave & 1;
    // kQuadForm: the tile rows with the longest k range are dispatched first
    const int tile_row = MODE == kQuadForm ? (int)(gridDim.y - 1 - blockIdx.y) : (int)blockIdx.y;
    const int r0 = tile_row * kTile, c0 = blockIdx.x * kTile;
    // loader: thread t brings rows t/32 and t/32 + 8 of a 16 x 128 tile, four floats at column 4 (t%32)
    const int lk = tid >> 5, lx = (tid & 31) * 4;

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    // kQuadForm: A is symmetric (the Hessian) and the caller wants sum_r E[r][c] C[r][c] with E = B, i.e.
    // b^T A b: the terms k > r are folded onto k < r (weight 2, diagonal 1), which halves the k range.
    const int Kend = MODE == kQuadForm ? (K < r0 + kTile ? K : r0 + kTile) : K;
    auto load_a = [&](int k) {
        f32x4v v = load4_or_zero(A, lda, k, Kend, r0 + lx, R);
        if (MODE == kQuadForm) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int r = r0 + lx + e;
                v[e] *= k < r ? 2.0f : (k == r ? 1.0f : 0.0f);
            }
        }
        return v;
    };
    f32x4v ra[2], rb[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        ra[h] = load_a(lk + 8 * h);
        rb[h] = load4_or_zero(B, ldb, lk + 8 * h, Kend, c0 + lx, C);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        *reinterpret_cast<f32x4v *>(&As[0][lk + 8 * h][lx]) = ra[h];
        *reinterpret_cast<f32x4v *>(&Bs[0][lk + 8 * h][lx]) = rb[h];
    }
    __syncthreads();
    int buf = 0;
    for (int k0 = 0; k0 < Kend; k0 += kStep) {
        const bool more = k0 + kStep < Kend;
        if (more) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                ra[h] = load_a(k0 + kStep + lk + 8 * h);
                rb[h] = load4_or_zero(B, ldb, k0 + kStep + lk + 8 * h, Kend, c0 + lx, C);
            }
        }
#pragma unroll
        for (int s = 0; s < kStep / 2; ++s) {
            const float a0 = As[buf][2 * s + hi][wr * 64 + lo], a1 = As[buf][2 * s + hi][wr * 64 + 32 + lo];
            const float b0 = Bs[buf][2 * s + hi][wc * 64 + lo], b1 = Bs[buf][2 * s + hi][wc * 64 + 32 + lo];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
        if (more) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                *reinterpret_cast<f32x4v *>(&As[buf ^ 1][lk + 8 * h][lx]) = ra[h];
                *reinterpret_cast<f32x4v *>(&Bs[buf ^ 1][lk + 8 * h][lx]) = rb[h];
            }
        }
        __syncthreads();  // the other buffer is complete, and everyone is done reading this one
        buf ^= 1;
    }

    // element i of a 32 x 32 accumulator: row 8 (i/4) + 4 hi + i%4, column lo
    if constexpr (MODE != kQuadForm) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int c = c0 + wc * 64 + b * 32 + lo;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int r = r0 + wr * 64 + a * 32 + 8 * (i >> 2) + 4 * hi + (i & 3);
                    if (r < R && c < C) {
                        float *o = out + (size_t)r * ldo + c;
                        if (MODE == kSubtract) *o -= acc[a][b][i];
                        if (MODE == kAddTwice) *o += 2.0f * acc[a][b][i];
                        if (MODE == kStore) *o = acc[a][b][i];
                        if (MODE == kStoreNegated) *o = -acc[a][b][i];
                    }
                }
            }
    } else {
        float *red = &As[0][0][0];  // [2 row halves][128 columns], free after the loop's last barrier
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int c = c0 + wc * 64 + b * 32 + lo;
            float sum = 0.0f;
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int r = r0 + wr * 64 + a * 32 + 8 * (i >> 2) + 4 * hi + (i & 3);
                    if (r < R && c < C) sum = fmaf(acc[a][b][i], E[(size_t)r * ldo + c], sum);
                }
            sum += __shfl_xor(sum, 32);
            if (hi == 0) red[wr * kTile + wc * 64 + b * 32 + lo] = sum;
        }
        __syncthreads();
        if (tid < kTile && c0 + tid < C) out[(size_t)tile_row * ldo + c0 + tid] = red[tid] + red[kTile + tid];
    }
}

// ---------------------------------------------------------------------------------
// Hessian of the layer-wise objective (Sec. II-A): H += 2 X^T X for T more calibration inputs
// ---------------------------------------------------------------------------------
hipError_t launch_quant_hessian(int N, int T, const float *X, float *H, hipStream_t stream)
{
    // X is [T][N]: k-major for both operands, C[r][c] = sum_t X[t][r] X[t][c]
    hipLaunchKernelGGL((mfma_kmajor_kernel<kAddTwice>), dim3((N + kTile - 1) / kTile, (N + kTile - 1) / kTile), dim3(256),
                       0, stream, X, N, N, X, N, N, T, H, N, nullptr);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// U with (H + lambda I)^-1 = U^T U, U upper triangular: what the GPTQ pass reads (Eq. 2)
// ---------------------------------------------------------------------------------
// With H_d = H + lambda I = R R^T, R UPPER triangular (a Cholesky factorisation taken from the last
// row upwards), H_d^-1 = R^-T R^-1, so U = R^-1.  Both steps are blocked by 128 columns; the diagonal
// blocks are factored and inverted by one workgroup in LDS, everything else is the k-major product
// above (K = 128 panels and trailing updates for R; growing K for the off-diagonal blocks of U).
// Working matrices (binary32, pitch N): Hw = H_d (consumed), Rt = R^T, Ut = U^T, T = one panel.
constexpr int kFactorBlock = 128;

__global__ void diag_mean_kernel(int N, const float *__restrict__ H, float damp, float *__restrict__ lambda)
{
    __shared__ float part[256];
    float s = 0.0f;
    for (int i = threadIdx.x; i < N; i += 256) s += H[(size_t)i * N + i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int k = 128; k > 0; k >>= 1) {
        if ((int)threadIdx.x < k) part[threadIdx.x] += part[threadIdx.x + k];
        __syncthreads();
    }
    if (threadIdx.x == 0) *lambda = damp * part[0] / (float)N;
}

__global__ void damped_copy_kernel(int N, const float *__restrict__ H, const float *__restrict__ lambda,
                                   float *__restrict__ Hw)
{
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (size_t)N * N) return;
    const int i = (int)(gid / N), j = (int)(gid - (size_t)i * N);
    Hw[gid] = H[gid] + (i == j ? *lambda : 0.0f);
}

// Diagonal block [r0, r0 + b): D = R R^T in place (R upper, from the last column to the first), then
// R^-1 beside it; writes the block of U and of U^T.  One workgroup; both blocks sit in LDS with an
// odd pitch so that rows and columns are both conflict-free.
constexpr int kDiagPitch = kFactorBlock + 1;
constexpr int kDiagLdsBytes = 2 * kFactorBlock * kDiagPitch * 4;  // the block and its inverse, 132096 B: dynamic

// Straight-line (no branch per element, so the LDS reads are issued together): every owned element of
// the first NM x NM groups is read, changed only where i <= l < j, and written back by its one owner.
template <int NM>
__device__ __forceinline__ void corner_update(float *D, int j, int ty, int tx)
{
    float ri[NM], rl[NM], v[NM][NM];
#pragma unroll
    for (int a = 0; a < NM; ++a) {
        ri[a] = D[(ty + 16 * a) * kDiagPitch + j];
        rl[a] = D[(tx + 16 * a) * kDiagPitch + j];
    }
#pragma unroll
    for (int a = 0; a < NM; ++a)
#pragma unroll
        for (int c = 0; c < NM; ++c) v[a][c] = D[(ty + 16 * a) * kDiagPitch + tx + 16 * c];
#pragma unroll
    for (int a = 0; a < NM; ++a)
#pragma unroll
        for (int c = 0; c < NM; ++c) {
            const int i = ty + 16 * a, l = tx + 16 * c;
            v[a][c] -= (i <= l && l < j) ? ri[a] * rl[c] : 0.0f;
        }
#pragma unroll
    for (int a = 0; a < NM; ++a)
#pragma unroll
        for (int c = 0; c < NM; ++c) D[(ty + 16 * a) * kDiagPitch + tx + 16 * c] = v[a][c];
}

__global__ __launch_bounds__(256) void factor_diag_kernel(int N, int r0, int b, const float *__restrict__ Hw,
                                                          float *__restrict__ U, float *__restrict__ Ut)
{
    extern __shared__ float D[];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    for (int e = tid; e < b * b; e += 256) {
        const int i = e / b, l = e - i * b;
        D[i * kDiagPitch + l] = Hw[(size_t)(r0 + i) * N + r0 + l];
    }
    __syncthreads();
    // column j of R = column j of the remaining block / sqrt(its corner); then the corner's rank-1 update.
    // D[j][j] keeps the un-rooted corner until the end (nobody reads it after step j).
    for (int j = b - 1; j >= 0; --j) {
        const float d = sqrtf(D[j * kDiagPitch + j]);
        if (tid < j) D[tid * kDiagPitch + j] /= d;  // own element: read and written by this thread only
        __syncthreads();
        // D[i][l] -= R[i][j] R[l][j] for i <= l < j; thread (ty, tx) owns i = ty + 16 a, l = tx + 16 c
        switch ((j + 15) >> 4) {  // uniform: how many 16 x 16 groups reach below j
            case 1: corner_update<1>(D, j, ty, tx); break;
            case 2: corner_update<2>(D, j, ty, tx); break;
            case 3: corner_update<3>(D, j, ty, tx); break;
            case 4: corner_update<4>(D, j, ty, tx); break;
            case 5: corner_update<5>(D, j, ty, tx); break;
            case 6: corner_update<6>(D, j, ty, tx); break;
            case 7: corner_update<7>(D, j, ty, tx); break;
            case 8: corner_update<8>(D, j, ty, tx); break;
            default: break;
        }
        __syncthreads();
    }
    if (tid < b) D[tid * kDiagPitch + tid] = sqrtf(D[tid * kDiagPitch + tid]);
    __syncthreads();
    // V = R^-1 into the second half of the LDS block, one thread per column and no barrier: column j of
    // R V = I from its diagonal upwards, v[i][j] = -(sum_{i < m <= j} r[i][m] v[m][j]) / r[i][i].  In step i
    // the threads read the same r[i][m] (broadcast) and their own column of V.
    float *V = D + kFactorBlock * kDiagPitch;
    if (tid < b) {
        const int j = tid;
        V[j * kDiagPitch + j] = 1.0f / D[j * kDiagPitch + j];
        for (int i = j - 1; i >= 0; --i) {
            float acc = 0.0f;
            for (int m = i + 1; m <= j; ++m) acc = fmaf(D[i * kDiagPitch + m], V[m * kDiagPitch + j], acc);
            V[i * kDiagPitch + j] = -acc / D[i * kDiagPitch + i];
        }
    }
    __syncthreads();
    for (int e = tid; e < b * b; e += 256) {
        const int i = e / b, l = e - i * b;
        const float v = i <= l ? V[i * kDiagPitch + l] : 0.0f;
        U[(size_t)(r0 + i) * N + r0 + l] = v;
        Ut[(size_t)(r0 + l) * N + r0 + i] = v;
    }
}

// dst[c][r] = src[r][c] for a rows x cols block.
__global__ void transpose_block_kernel(int rows, int cols, const float *__restrict__ src, int lds, float *__restrict__ dst,
                                       int ldd)
{
    __shared__ float tile[32][33];
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    for (int i = threadIdx.y; i < 32; i += blockDim.y) {
        const int r = r0 + i, c = c0 + threadIdx.x;
        tile[i][threadIdx.x] = (r < rows && c < cols) ? src[(size_t)r * lds + c] : 0.0f;
    }
    __syncthreads();
    for (int i = threadIdx.y; i < 32; i += blockDim.y) {
        const int c = c0 + i, r = r0 + threadIdx.x;
        if (r < rows && c < cols) dst[(size_t)c * ldd + r] = tile[threadIdx.x][i];
    }
}

size_t quant_factor_workspace_bytes(int N)
{
    const size_t floats = 3 * (size_t)N * N + 64;
    return (floats * 4 + 255) / 256 * 256;
}

template <int MODE>
static void product(hipStream_t stream, const float *A, int lda, int R, const float *B, int ldb, int C, int K, float *out,
                    int ldo)
{
    hipLaunchKernelGGL((mfma_kmajor_kernel<MODE>), dim3((C + kTile - 1) / kTile, (R + kTile - 1) / kTile), dim3(256), 0,
                       stream, A, lda, R, B, ldb, C, K, out, ldo, nullptr);
}

// Off-diagonal blocks of U = R^-1 for the rows / columns [lo, hi) (the diagonal blocks are in place):
// with the range cut at a block boundary, U12 = -U11 (R12 U22), both factors from the two halves.
static void invert_range(hipStream_t stream, int N, int lo, int hi, const float *Rt, float *U, float *Ut, float *T)
{
    const int nblk = (hi - lo + kFactorBlock - 1) / kFactorBlock;
    if (nblk <= 1) return;
    const int mid = lo + (nblk / 2) * kFactorBlock;
    invert_range(stream, N, lo, mid, Rt, U, Ut, T);
    invert_range(stream, N, mid, hi, Rt, U, Ut, T);
    const int rows = mid - lo, cols = hi - mid;
    // T[i][c] = sum_m R[lo + i][mid + m] U[mid + m][mid + c]
    product<kStore>(stream, Rt + (size_t)mid * N + lo, N, rows, U + (size_t)mid * N + mid, N, cols, cols, T, cols);
    // U[lo + r][mid + c] = -sum_j U[lo + r][lo + j] T[j][c]
    product<kStoreNegated>(stream, Ut + (size_t)lo * N + lo, N, rows, T, cols, cols, rows, U + (size_t)lo * N + mid, N);
    hipLaunchKernelGGL(transpose_block_kernel, dim3((cols + 31) / 32, (rows + 31) / 32), dim3(32, 8), 0, stream, rows, cols,
                       U + (size_t)lo * N + mid, N, Ut + (size_t)mid * N + lo, N);
}

hipError_t launch_quant_factor(int N, float damp, const float *H, float *U, void *workspace, hipStream_t stream)
{
    float *Hw = static_cast<float *>(workspace);
    float *Rt = Hw + (size_t)N * N, *Ut = Rt + (size_t)N * N;
    float *lambda = Ut + (size_t)N * N;
    static bool lds_set = false;  // per process; the attribute belongs to the function, not to a device
    if (!lds_set) {
        hipError_t a = hipFuncSetAttribute(reinterpret_cast<const void *>(factor_diag_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kDiagLdsBytes);
        if (a != hipSuccess) return a;
        lds_set = true;
    }
    hipLaunchKernelGGL(diag_mean_kernel, dim3(1), dim3(256), 0, stream, N, H, damp, lambda);
    hipLaunchKernelGGL(damped_copy_kernel, dim3((unsigned)(((size_t)N * N + 255) / 256)), dim3(256), 0, stream, N, H,
                       lambda, Hw);
    hipError_t e = launch_fill_zero(U, (size_t)N * N * 4, stream);
    if (e != hipSuccess) return e;
    e = launch_fill_zero(Ut, (size_t)N * N * 4, stream);
    if (e != hipSuccess) return e;
    const int nblk = (N + kFactorBlock - 1) / kFactorBlock;
    // R, from the last block column to the first
    for (int k = nblk - 1; k >= 0; --k) {
        const int r0 = k * kFactorBlock, b = N - r0 < kFactorBlock ? N - r0 : kFactorBlock;
        hipLaunchKernelGGL(factor_diag_kernel, dim3(1), dim3(256), kDiagLdsBytes, stream, N, r0, b, Hw, U, Ut);
        if (r0 == 0) break;
        // panel, transposed: Rt[r0 + c][i] = R[i][r0 + c] = sum_m V[c][m] Hw[r0 + m][i]   (Hw symmetric, V = R_kk^-1)
        product<kStore>(stream, Ut + (size_t)r0 * N + r0, N, b, Hw + (size_t)r0 * N, N, r0, b, Rt + (size_t)r0 * N, N);
        // Hw[i][j] -= sum_c R[i][r0 + c] R[j][r0 + c] for i, j < r0
        product<kSubtract>(stream, Rt + (size_t)r0 * N, N, r0, Rt + (size_t)r0 * N, N, r0, b, Hw, N);
    }
    // U = R^-1: Hw is free now and holds the intermediate products
    invert_range(stream, N, 0, N, Rt, U, Ut, Hw);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// search
// ---------------------------------------------------------------------------------
// Row minimum and maximum in two steps: `chunks` slabs of columns each leave a partial pair in
// scratch ([chunks][Mp] minima, then [chunks][Mp] maxima), a second launch combines them.
__global__ void row_range_partial_kernel(int M, int Mp, int N, int chunks, const float *__restrict__ Wt,
                                         float *__restrict__ scratch)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x, chunk = blockIdx.y;
    if (m >= M) return;
    const int per = (N + chunks - 1) / chunks;
    const int k_end = (chunk + 1) * per < N ? (chunk + 1) * per : N;
    float lo = INFINITY, hi = -INFINITY;
    for (int k = chunk * per; k < k_end; ++k) {
        const float v = Wt[(size_t)k * Mp + m];
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
    scratch[(size_t)chunk * Mp + m] = lo;
    scratch[(size_t)(chunks + chunk) * Mp + m] = hi;
}

__global__ void row_range_final_kernel(int M, int Mp, int chunks, const float *__restrict__ scratch,
                                       float *__restrict__ wmin, float *__restrict__ wmax)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= M) return;
    float lo = INFINITY, hi = -INFINITY;
    for (int c = 0; c < chunks; ++c) {
        lo = fminf(lo, scratch[(size_t)c * Mp + m]);
        hi = fmaxf(hi, scratch[(size_t)(chunks + c) * Mp + m]);
    }
    wmin[m] = lo;
    wmax[m] = hi;
}

// Scale of grid point g (0-based) of a row, Eq. 7, in binary64.
__device__ __forceinline__ double grid_scale(double wmin, double wmax, int n_bits, int g, int grid)
{
    if (wmax == wmin) return 1.0;  // a constant row: Eq. 7's interval is empty, any scale reproduces it
    const double lo = (wmax - wmin) / (double)((1 << (n_bits + 1)) - 1);
    const double hi = (wmax - wmin) / (double)((1 << (n_bits - 1)) - 1);
    return lo + (hi - lo) * ((double)(g + 1) / ((double)grid + 1.0));
}

// Dt[k][m] = S' W_q + qbias - w for one candidate (grid point g, tying t); zeros in the pad rows.
__global__ void delta_kernel(int M, int Mp, int N, int n_bits, int g, int grid, Tying t,
                             const float *__restrict__ Wt, const float *__restrict__ wmin,
                             const float *__restrict__ wmax, float *__restrict__ Dt)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = blockIdx.y;
    if (m >= Mp) return;
    float d = 0.0f;
    if (m < M) {
        const double lo = wmin[m], S = grid_scale(lo, wmax[m], n_bits, g, grid);
        const double w = Wt[(size_t)k * Mp + m];
        const int wq = quant_int(w, S, lo, n_bits, t.choice, t.nchoice);
        d = (float)(S * wq + lo - w);
    }
    Dt[(size_t)k * Mp + m] = d;
}

// err = (sum of the row's tile partials, in tile order) / 2 (H = 2 X X^T); keep the candidate if it
// is strictly better.
__global__ void keep_best_kernel(int M, int Mp, int n_bits, int ntile, int g, int grid, int first, Tying t,
                                 const float *__restrict__ part, const float *__restrict__ wmin,
                                 const float *__restrict__ wmax, float *__restrict__ best, float *__restrict__ S,
                                 float *__restrict__ qbias, int8_t *__restrict__ labels)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= M) return;
    float e = 0.0f;
    for (int k = 0; k < ntile; ++k) e += part[(size_t)k * Mp + m];
    e *= 0.5f;
    if (first || e < best[m]) {
        best[m] = e;
        S[m] = (float)grid_scale(wmin[m], wmax[m], n_bits, g, grid);
        qbias[m] = wmin[m];
        for (int i = 0; i < n_bits; ++i) labels[(size_t)m * n_bits + i] = t.label[i];
    }
}

hipError_t launch_quant_search(int M, int N, int n_bits, int q, int grid, const float *W, const float *H, float *S,
                               float *qbias, int8_t *labels, float *err_out, void *workspace, hipStream_t stream)
{
    const QuantWorkspace w = carve(workspace, M, N);
    hipLaunchKernelGGL(transpose_kernel, dim3((N + 31) / 32, (w.Mp + 31) / 32), dim3(32, 8), 0, stream, M, w.Mp, N, W,
                       w.Wt);
    const int chunks = N / 2 < 64 ? N / 2 : 64;  // Dt (N rows, not yet in use) holds the 2 * chunks partial rows
    hipLaunchKernelGGL(row_range_partial_kernel, dim3((M + 63) / 64, chunks), dim3(64), 0, stream, M, w.Mp, N, chunks,
                       w.Wt, w.Dt);
    hipLaunchKernelGGL(row_range_final_kernel, dim3((M + 63) / 64), dim3(64), 0, stream, M, w.Mp, chunks, w.Dt, w.wmin,
                       w.wmax);
    const std::vector<Tying> tyings = all_tyings(n_bits, q);
    bool first = true;
    for (int g = 0; g < grid; ++g)
        for (const Tying &t : tyings) {
            hipLaunchKernelGGL(delta_kernel, dim3((w.Mp + 255) / 256, N), dim3(256), 0, stream, M, w.Mp, N, n_bits, g,
                               grid, t, w.Wt, w.wmin, w.wmax, w.Dt);
            // d H d^T row by row: sum_l Dt[l][m] sum_{k <= l} w_kl H[k][l] Dt[k][m], w = 2 off the diagonal
            // (only the upper triangle of H is read), one partial per tile of 128 values of l
            hipLaunchKernelGGL((mfma_kmajor_kernel<kQuadForm>), dim3((w.Mp + kTile - 1) / kTile, w.ntile), dim3(256), 0,
                               stream, H, N, N, w.Dt, w.Mp, w.Mp, N, w.part, w.Mp, w.Dt);
            hipLaunchKernelGGL(keep_best_kernel, dim3((M + 255) / 256), dim3(256), 0, stream, M, w.Mp, n_bits, w.ntile, g,
                               grid, first ? 1 : 0, t, w.part, w.wmin, w.wmax, w.best, S, qbias, labels);
            first = false;
        }
    if (err_out) {
        hipError_t e = hipMemcpyAsync(err_out, w.best, (size_t)M * 4, hipMemcpyDeviceToDevice, stream);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// GPTQ pass
// ---------------------------------------------------------------------------------
// One block of up to 128 columns [c0, c1): one thread per row.  The block's columns of the row sit in
// LDS; the 32 columns being decided are held in registers, where each decision's compensation reaches
// the later ones of the 32 at once, and reach the block's remaining columns when the 32 are done
// (the same order of operations per weight as column by column).  The rows of U that the 32 columns
// need are staged in LDS: the 32 x 32 corner as it is, the part to its right transposed so that one
// column's 32 factors are contiguous.
constexpr int kGptqBlock = 128, kGptqRows = 64, kGptqSub = 32;
__global__ __launch_bounds__(kGptqRows) void gptq_block_kernel(int M, int Mp, int N, int n_bits, int q, int c0, int c1,
                                                               float *__restrict__ Wt, const float *__restrict__ U,
                                                               const float *__restrict__ S, const float *__restrict__ qbias,
                                                               const int8_t *__restrict__ labels,
                                                               uint8_t *__restrict__ w_int, float *__restrict__ Err)
{
    __shared__ float wl[kGptqBlock][kGptqRows + 1];
    __shared__ __attribute__((aligned(16))) float Ud[kGptqSub][kGptqSub];
    __shared__ __attribute__((aligned(16))) float Uo[kGptqBlock - kGptqSub][kGptqSub];
    const int tm = threadIdx.x, m = blockIdx.x * kGptqRows + tm;
    const bool live = m < M;
    const int cols = c1 - c0;
    int choice[16];
    double s = 1.0, b = 0.0;
    if (live) {
        TyingPlan plan;  // labels come from device memory the host cannot inspect: out-of-range ones are folded
        make_tying_plan(n_bits, q, labels + (size_t)m * n_bits, true, &plan);
        for (int k = 0; k < 16; ++k) choice[k] = plan.choice[k];
        s = S[m]; b = qbias[m];
    }
    for (int j = 0; j < cols; ++j) wl[j][tm] = live ? Wt[(size_t)(c0 + j) * Mp + m] : 0.0f;
    for (int sb = 0; sb < cols; sb += kGptqSub) {
        const int sw = cols - sb < kGptqSub ? cols - sb : kGptqSub;
        const int rest = cols - sb - sw;
        __syncthreads();  // the previous round's readers of Ud / Uo are done
        for (int e = tm; e < kGptqSub * kGptqSub; e += kGptqRows) {
            const int i = e >> 5, k = e & 31;
            Ud[i][k] = (i < sw && k < sw) ? U[(size_t)(c0 + sb + i) * N + c0 + sb + k] : (i == k ? 1.0f : 0.0f);
        }
        for (int e = tm; e < rest * kGptqSub; e += kGptqRows) {
            const int i = e / rest, k = e - i * rest;
            Uo[k][i] = U[(size_t)(c0 + sb + i) * N + c0 + sb + sw + k];  // rest > 0 only with sw = 32
        }
        __syncthreads();
        float w[kGptqSub], err[kGptqSub];
#pragma unroll
        for (int i = 0; i < kGptqSub; ++i) w[i] = i < sw ? wl[sb + i][tm] : 0.0f;
#pragma unroll
        for (int i = 0; i < kGptqSub; ++i) {
            err[i] = 0.0f;
            if (i < sw) {  // uniform
                if (live) {
                    const int wq = quant_int((double)w[i], s, b, n_bits, choice, 1 << q);
                    w_int[(size_t)m * N + c0 + sb + i] = (uint8_t)wq;
                    const float qv = (float)(s * wq + b);
                    err[i] = (w[i] - qv) / Ud[i][i];
                }
                if (m < Mp) Err[(size_t)(sb + i) * Mp + m] = err[i];  // zeros in the pad rows
#pragma unroll
                for (int k = i + 1; k < kGptqSub; ++k) w[k] = fmaf(-err[i], Ud[i][k], w[k]);
            }
        }
        for (int k = 0; k < rest; ++k) {
            float a = wl[sb + sw + k][tm];
#pragma unroll
            for (int i = 0; i < kGptqSub; ++i) a = fmaf(-err[i], Uo[k][i], a);
            wl[sb + sw + k][tm] = a;
        }
    }
}

hipError_t launch_quant_gptq(int M, int N, int n_bits, int q, const float *W, const float *U, const float *S,
                             const float *qbias, const int8_t *labels, uint8_t *w_int, void *workspace,
                             hipStream_t stream)
{
    const QuantWorkspace w = carve(workspace, M, N);
    hipLaunchKernelGGL(transpose_kernel, dim3((N + 31) / 32, (w.Mp + 31) / 32), dim3(32, 8), 0, stream, M, w.Mp, N, W,
                       w.Wt);
    for (int c0 = 0; c0 < N; c0 += kGptqBlock) {
        const int c1 = c0 + kGptqBlock < N ? c0 + kGptqBlock : N;
        hipLaunchKernelGGL(gptq_block_kernel, dim3((w.Mp + kGptqRows - 1) / kGptqRows), dim3(kGptqRows), 0, stream, M,
                           w.Mp, N, n_bits, q, c0, c1, w.Wt, U, S, qbias, labels, w_int, w.Err);
        if (c1 < N)  // Wt[k][m] -= sum_j U[c0 + j][k] Err[j][m] for the columns k >= c1
            hipLaunchKernelGGL((mfma_kmajor_kernel<kSubtract>), dim3((w.Mp + kTile - 1) / kTile, (N - c1 + kTile - 1) / kTile),
                               dim3(256), 0, stream, U + (size_t)c0 * N + c1, N, N - c1, w.Err, w.Mp, w.Mp, c1 - c0,
                               w.Wt + (size_t)c1 * w.Mp, w.Mp, nullptr);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// fusion with one tying per row (row-wise parameters: one scaling group per row)
// ---------------------------------------------------------------------------------
__global__ void from_linear_rows_kernel(int M, int N, int n_bits, int q, const int8_t *__restrict__ labels,
                                        const uint8_t *__restrict__ w_int, const float *__restrict__ S,
                                        const float *__restrict__ qbias, uint8_t *__restrict__ codes,
                                        uint16_t *__restrict__ alpha, uint16_t *__restrict__ offset)
{
    const int m = blockIdx.x;
    __shared__ TyingPlan plan;
    if (threadIdx.x == 0) {
        make_tying_plan(n_bits, q, labels + (size_t)m * n_bits, true, &plan);
        const double s = S[m];
        for (int o = 0; o < q; ++o) alpha[(size_t)m * q + o] = double_to_half_bits(s * plan.alpha_hat[o]);
        offset[m] = double_to_half_bits(((1 << n_bits) - 1) / 2.0 * s + (double)qbias[m]);
    }
    __syncthreads();
    for (int k = threadIdx.x; k < N; k += blockDim.x) {
        const int w = w_int[(size_t)m * N + k] & ((1 << n_bits) - 1);
        codes[(size_t)m * N + k] = code_of(nearest_choice(w, plan.choice, plan.nchoice), plan, q);  // Eq. 6 (members pass unchanged)
    }
}

hipError_t launch_from_linear_rows(int M, int N, int n_bits, int q, const int8_t *labels, const uint8_t *w_int,
                                   const float *S, const float *qbias, uint8_t *codes, uint16_t *alpha,
                                   uint16_t *offset, hipStream_t stream)
{
    hipLaunchKernelGGL(from_linear_rows_kernel, dim3(M), dim3(256), 0, stream, M, N, n_bits, q, labels, w_int, S, qbias,
                       codes, alpha, offset);
    return hipGetLastError();
}

}  // namespace bcq
