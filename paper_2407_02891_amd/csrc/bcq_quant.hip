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

namespace bcq {

constexpr int kMaxBits = 8;

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
        t.nchoice = 1 << q;
        for (int m = 0; m < t.nchoice; ++m) {
            int v = 0;
            for (int i = 0; i < n; ++i)
                if ((m >> t.label[i]) & 1) v |= 1 << i;
            t.choice[m] = v;
        }
        std::sort(t.choice, t.choice + t.nchoice);
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
    const int wi = (int)v;
    int best = choice[0], best_d = abs(wi - choice[0]);
    for (int k = 1; k < nchoice; ++k) {
        const int d = abs(wi - choice[k]);
        if (d < best_d) { best_d = d; best = choice[k]; }  // strict: the smaller member on a tie
    }
    return best;
}

// ---------------------------------------------------------------------------------
// search
// ---------------------------------------------------------------------------------
__global__ void row_range_kernel(int M, int N, const float *__restrict__ W, float *__restrict__ wmin,
                                 float *__restrict__ wmax)
{
    const int m = blockIdx.x;
    float lo = INFINITY, hi = -INFINITY;
    for (int k = threadIdx.x; k < N; k += blockDim.x) {
        const float v = W[(size_t)m * N + k];
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
    __shared__ float slo[256], shi[256];
    slo[threadIdx.x] = lo; shi[threadIdx.x] = hi;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            slo[threadIdx.x] = fminf(slo[threadIdx.x], slo[threadIdx.x + s]);
            shi[threadIdx.x] = fmaxf(shi[threadIdx.x], shi[threadIdx.x + s]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) { wmin[m] = slo[0]; wmax[m] = shi[0]; }
}

// Scale of grid point g (0-based) of a row, Eq. 7, in binary64.
__device__ __forceinline__ double grid_scale(double wmin, double wmax, int n_bits, int g, int grid)
{
    const double lo = (wmax - wmin) / (double)((1 << (n_bits + 1)) - 1);
    const double hi = (wmax - wmin) / (double)((1 << (n_bits - 1)) - 1);
    return lo + (hi - lo) * ((double)(g + 1) / ((double)grid + 1.0));
}

// D[m][k] = S' W_q + qbias - w for one candidate (grid point g, tying t).
__global__ void delta_kernel(int M, int N, int n_bits, int g, int grid, Tying t, const float *__restrict__ W,
                             const float *__restrict__ wmin, const float *__restrict__ wmax, float *__restrict__ D)
{
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (size_t)M * N) return;
    const int m = (int)(gid / N);
    const double lo = wmin[m], S = grid_scale(lo, wmax[m], n_bits, g, grid);
    const double w = W[gid];
    const int wq = quant_int(w, S, lo, n_bits, t.choice, t.nchoice);
    D[gid] = (float)(S * wq + lo - w);
}

// part[m][tile] = sum over the 64 columns l of the tile of D[m][l] * (sum_k D[m][k] H[k][l]).
constexpr int kBM = 64, kBN = 64, kBK = 16;
__global__ __launch_bounds__(256) void quad_form_kernel(int M, int N, const float *__restrict__ D,
                                                        const float *__restrict__ H, float *__restrict__ part,
                                                        int ntile)
{
    __shared__ float As[kBK][kBM + 1];
    __shared__ float Bs[kBK][kBN];
    __shared__ float red[kBM][17];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int l0 = blockIdx.x * kBN, m0 = blockIdx.y * kBM;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < N; k0 += kBK) {
        for (int e = tid; e < kBM * kBK; e += 256) {  // D tile, 64 rows x 16 k
            const int mm = e / kBK, kk = e % kBK;
            const int m = m0 + mm, k = k0 + kk;
            As[kk][mm] = (m < M && k < N) ? D[(size_t)m * N + k] : 0.0f;
        }
        for (int e = tid; e < kBK * kBN; e += 256) {  // H tile, 16 k x 64 l
            const int kk = e / kBN, ll = e % kBN;
            const int k = k0 + kk, l = l0 + ll;
            Bs[kk][ll] = (k < N && l < N) ? H[(size_t)k * N + l] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kBK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        float s = 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int l = l0 + tx * 4 + j;
            if (m < M && l < N) s = fmaf(acc[i][j], D[(size_t)m * N + l], s);
        }
        red[ty * 4 + i][tx] = s;
    }
    __syncthreads();
    if (tid < kBM) {  // fixed order: the result does not depend on timing
        float s = 0.0f;
        for (int t = 0; t < 16; ++t) s += red[tid][t];
        const int m = m0 + tid;
        if (m < M) part[(size_t)m * ntile + blockIdx.x] = s;
    }
}

// err = (sum of the row's tile partials) / 2 (H = 2 X X^T); keep the candidate if it is strictly better.
__global__ void keep_best_kernel(int M, int n_bits, int ntile, int g, int grid, int first, Tying t,
                                 const float *__restrict__ part, const float *__restrict__ wmin,
                                 const float *__restrict__ wmax, float *__restrict__ best, float *__restrict__ S,
                                 float *__restrict__ qbias, int8_t *__restrict__ labels)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= M) return;
    float e = 0.0f;
    for (int k = 0; k < ntile; ++k) e += part[(size_t)m * ntile + k];
    e *= 0.5f;
    if (first || e < best[m]) {
        best[m] = e;
        S[m] = (float)grid_scale(wmin[m], wmax[m], n_bits, g, grid);
        qbias[m] = wmin[m];
        for (int i = 0; i < n_bits; ++i) labels[(size_t)m * n_bits + i] = t.label[i];
    }
}

size_t quant_workspace_bytes(int M, int N)
{
    const size_t ntile = (size_t)(N + kBN - 1) / kBN;
    size_t floats = (size_t)M * N          // D, later the transposed working copy of W
                    + (size_t)M * ntile    // tile partials
                    + 3 * (size_t)M        // row min, row max, best error
                    + 128 * (size_t)M;     // GPTQ: errors of one block of columns
    return (floats * 4 + 255) / 256 * 256;
}

hipError_t launch_quant_search(int M, int N, int n_bits, int q, int grid, const float *W, const float *H, float *S,
                               float *qbias, int8_t *labels, float *err_out, void *workspace, hipStream_t stream)
{
    const int ntile = (N + kBN - 1) / kBN;
    float *D = static_cast<float *>(workspace);
    float *part = D + (size_t)M * N;
    float *wmin = part + (size_t)M * ntile, *wmax = wmin + M, *best = wmax + M;
    hipLaunchKernelGGL(row_range_kernel, dim3(M), dim3(256), 0, stream, M, N, W, wmin, wmax);
    const std::vector<Tying> tyings = all_tyings(n_bits, q);
    const size_t total = (size_t)M * N;
    bool first = true;
    for (int g = 0; g < grid; ++g)
        for (const Tying &t : tyings) {
            hipLaunchKernelGGL(delta_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, M, N, n_bits,
                               g, grid, t, W, wmin, wmax, D);
            hipLaunchKernelGGL(quad_form_kernel, dim3(ntile, (M + kBM - 1) / kBM), dim3(256), 0, stream, M, N, D, H,
                               part, ntile);
            hipLaunchKernelGGL(keep_best_kernel, dim3((M + 255) / 256), dim3(256), 0, stream, M, n_bits, ntile, g, grid,
                               first ? 1 : 0, t, part, wmin, wmax, best, S, qbias, labels);
            first = false;
        }
    if (err_out) {
        hipError_t e = hipMemcpyAsync(err_out, best, (size_t)M * 4, hipMemcpyDeviceToDevice, stream);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// GPTQ pass
// ---------------------------------------------------------------------------------
// Labels come from device memory the host cannot inspect: out-of-range ones are folded into 0..q-1.
__device__ __forceinline__ int class_of(const int8_t *label, int i, int q)
{
    const int c = label[i];
    return c < 0 ? 0 : (c >= q ? q - 1 : c);
}

// BCchoice of a row from its class labels (ascending).
__device__ __forceinline__ void row_choice(const int8_t *label, int n_bits, int q, int *choice)
{
    const int nc = 1 << q;
    for (int m = 0; m < nc; ++m) {
        int v = 0;
        for (int i = 0; i < n_bits; ++i)
            if ((m >> class_of(label, i, q)) & 1) v |= 1 << i;
        choice[m] = v;
    }
    for (int a = 1; a < nc; ++a) {  // insertion sort
        const int v = choice[a];
        int b = a - 1;
        while (b >= 0 && choice[b] > v) { choice[b + 1] = choice[b]; --b; }
        choice[b + 1] = v;
    }
}

__global__ void transpose_kernel(int M, int N, const float *__restrict__ W, float *__restrict__ Wt)
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
        if (m < M && k < N) Wt[(size_t)k * M + m] = tile[threadIdx.x][i];
    }
}

// One block of up to 128 columns [c0, c1): one thread per row, the block's columns of the row in LDS.
constexpr int kGptqBlock = 128, kGptqRows = 64;
__global__ __launch_bounds__(kGptqRows) void gptq_block_kernel(int M, int N, int n_bits, int q, int c0, int c1,
                                                               float *__restrict__ Wt, const float *__restrict__ U,
                                                               const float *__restrict__ S, const float *__restrict__ qbias,
                                                               const int8_t *__restrict__ labels,
                                                               uint8_t *__restrict__ w_int, float *__restrict__ Err)
{
    __shared__ float wl[kGptqBlock][kGptqRows + 1];
    const int tm = threadIdx.x, m = blockIdx.x * kGptqRows + tm;
    const bool live = m < M;
    const int cols = c1 - c0;
    int choice[16];
    double s = 1.0, b = 0.0;
    if (live) {
        row_choice(labels + (size_t)m * n_bits, n_bits, q, choice);
        s = S[m]; b = qbias[m];
    }
    for (int j = 0; j < cols; ++j) wl[j][tm] = live ? Wt[(size_t)(c0 + j) * M + m] : 0.0f;
    for (int j = 0; j < cols; ++j) {
        const int c = c0 + j;
        const float w = wl[j][tm];
        float e = 0.0f;
        if (live) {
            const int wq = quant_int((double)w, s, b, n_bits, choice, 1 << q);
            w_int[(size_t)m * N + c] = (uint8_t)wq;
            const float qv = (float)(s * wq + b);
            e = (w - qv) / U[(size_t)c * N + c];
        }
        if (live) Err[(size_t)j * M + m] = e;
        for (int k = j + 1; k < cols; ++k) wl[k][tm] = fmaf(-e, U[(size_t)c * N + c0 + k], wl[k][tm]);
    }
}

// Wt[k][m] -= sum_j Err[j][m] U[c0 + j][k] for the columns k >= c1.
__global__ void gptq_trailing_kernel(int M, int N, int c0, int c1, float *__restrict__ Wt, const float *__restrict__ U,
                                     const float *__restrict__ Err)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = c1 + blockIdx.y;
    if (m >= M || k >= N) return;
    float acc = 0.0f;
    for (int j = 0; j < c1 - c0; ++j) acc = fmaf(Err[(size_t)j * M + m], U[(size_t)(c0 + j) * N + k], acc);
    Wt[(size_t)k * M + m] -= acc;
}

hipError_t launch_quant_gptq(int M, int N, int n_bits, int q, const float *W, const float *U, const float *S,
                             const float *qbias, const int8_t *labels, uint8_t *w_int, void *workspace,
                             hipStream_t stream)
{
    const int ntile = (N + kBN - 1) / kBN;
    float *Wt = static_cast<float *>(workspace);
    float *Err = Wt + (size_t)M * N + (size_t)M * ntile + 3 * (size_t)M;
    hipLaunchKernelGGL(transpose_kernel, dim3((N + 31) / 32, (M + 31) / 32), dim3(32, 8), 0, stream, M, N, W, Wt);
    for (int c0 = 0; c0 < N; c0 += kGptqBlock) {
        const int c1 = c0 + kGptqBlock < N ? c0 + kGptqBlock : N;
        hipLaunchKernelGGL(gptq_block_kernel, dim3((M + kGptqRows - 1) / kGptqRows), dim3(kGptqRows), 0, stream, M, N,
                           n_bits, q, c0, c1, Wt, U, S, qbias, labels, w_int, Err);
        if (c1 < N)
            hipLaunchKernelGGL(gptq_trailing_kernel, dim3((M + 255) / 256, N - c1), dim3(256), 0, stream, M, N, c0, c1,
                               Wt, U, Err);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// fusion with one tying per row (row-wise parameters: one scaling group per row)
// ---------------------------------------------------------------------------------
__device__ __forceinline__ uint16_t double_to_half_bits_rne(double v)
{
    float f = __double2float_rz(v);
    if (static_cast<double>(f) != v && !(v != v)) f = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, f) | 1u);
    return float_to_half_bits(f);
}

// Per row: alpha_hat of every class, classes ordered by descending alpha_hat, the bit each output
// plane reads its sign from.
__device__ __forceinline__ void row_plan(const int8_t *label, int n_bits, int q, double *ah_sorted, int *sign_bit)
{
    double ah[kMaxQ] = {0, 0, 0, 0};
    int first[kMaxQ] = {-1, -1, -1, -1};
    for (int i = 0; i < n_bits; ++i) {
        const int c = class_of(label, i, q);
        ah[c] += (double)(1 << i) / 2.0;
        if (first[c] < 0) first[c] = i;
    }
    int order[kMaxQ] = {0, 1, 2, 3};
    for (int a = 0; a < q; ++a)
        for (int b = a + 1; b < q; ++b)
            if (ah[order[b]] > ah[order[a]]) { const int t = order[a]; order[a] = order[b]; order[b] = t; }
    for (int o = 0; o < q; ++o) { ah_sorted[o] = ah[order[o]]; sign_bit[o] = first[order[o]] < 0 ? 0 : first[order[o]]; }
}

__global__ void from_linear_rows_kernel(int M, int N, int n_bits, int q, const int8_t *__restrict__ labels,
                                        const uint8_t *__restrict__ w_int, const float *__restrict__ S,
                                        const float *__restrict__ qbias, uint8_t *__restrict__ codes,
                                        uint16_t *__restrict__ alpha, uint16_t *__restrict__ offset)
{
    const int m = blockIdx.x;
    __shared__ int sign_bit[kMaxQ];
    __shared__ int choice[16];
    if (threadIdx.x == 0) {
        double ah[kMaxQ];
        row_plan(labels + (size_t)m * n_bits, n_bits, q, ah, sign_bit);
        row_choice(labels + (size_t)m * n_bits, n_bits, q, choice);
        const double s = S[m];
        for (int o = 0; o < q; ++o) alpha[(size_t)m * q + o] = double_to_half_bits_rne(s * ah[o]);
        offset[m] = double_to_half_bits_rne(((1 << n_bits) - 1) / 2.0 * s + (double)qbias[m]);
    }
    __syncthreads();
    for (int k = threadIdx.x; k < N; k += blockDim.x) {
        const int w = w_int[(size_t)m * N + k] & ((1 << n_bits) - 1);
        int best = choice[0], best_d = abs(w - choice[0]);  // Eq. 6 (members pass unchanged)
        for (int c = 1; c < (1 << q); ++c) {
            const int d = abs(w - choice[c]);
            if (d < best_d) { best_d = d; best = choice[c]; }
        }
        uint8_t code = 0;
        for (int o = 0; o < q; ++o) code |= (uint8_t)(((best >> sign_bit[o]) & 1) << o);
        codes[(size_t)m * N + k] = code;
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
