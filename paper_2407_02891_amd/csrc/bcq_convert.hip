// bcq_from_linear: the step right before the hot path.  The two-step quantiser of the paper
// ends with n-bit linear integers W_int, a scale S and a bias qbias per scaling group, and a
// choice of which linear bit-planes are tied together (Sec. II-B, Eq. 6; Sec. II-D, Eq. 8-11).
// This turns them into the operands of Eq. 11 -- per-weight plane codes, fused alpha_hat,
// fused offset -- i.e. exactly what bcq_pack consumes.  Offline step; written for clarity.
//
//   Eq. 9   W_int = sum_{i=1..n} 2^(i-2) b_i + (2^n - 1)/2,  b_i = +1 iff bit i-1 of W_int is set
//   Eq. 10  tying the planes of a class c to one sign gives alpha_hat_c = sum_{i in c} 2^(i-2);
//           the integers reachable that way are BCchoice
//   Eq. 6   every W_int is replaced by the nearest member of BCchoice
//   Eq. 11  W_hat = sum_c (S alpha_hat_c) b_c + ((2^n - 1)/2 S + qbias)
#include "bcq_internal.h"
#include "bcq_device.h"

namespace bcq {

struct ConvertPlan {
    int n_bits, q;
    int nchoice;           // 2^q
    int choice[16];        // members of BCchoice, ascending
    int sign_bit[kMaxQ];   // output plane o takes its sign from this bit of the rounded integer
    double alpha_hat[kMaxQ];  // sum of 2^(i-2) over the planes tied into output plane o, descending
    double centre;         // (2^n - 1) / 2
};

// binary64 -> binary16, round to nearest even, with a single rounding: the value is first
// rounded to binary32 *to odd* (truncate, then set the last bit if anything was lost), which
// keeps enough information for the final rounding to be the correct one.
__device__ __forceinline__ uint16_t double_to_half_bits(double v)
{
    float f = __double2float_rz(v);
    if (static_cast<double>(f) != v && !(v != v)) {
        uint32_t u = __builtin_bit_cast(uint32_t, f);
        // |f| <= |v|: bump the magnitude's last bit when the truncation lost something (sticky bit)
        u |= 1u;
        f = __builtin_bit_cast(float, u);
    }
    return float_to_half_bits(f);
}

__global__ void from_linear_codes_kernel(ConvertPlan plan, const uint8_t *__restrict__ w_int,
                                         uint8_t *__restrict__ codes, size_t total)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int w = w_int[gid] & ((1 << plan.n_bits) - 1);
    // Eq. 6: nearest member of BCchoice; scanning upwards with a strict comparison keeps the
    // smaller member on a tie
    int best = plan.choice[0], best_d = abs(w - plan.choice[0]);
    for (int k = 1; k < plan.nchoice; ++k) {
        const int d = abs(w - plan.choice[k]);
        if (d < best_d) { best_d = d; best = plan.choice[k]; }
    }
    uint8_t code = 0;
    for (int o = 0; o < plan.q; ++o) code |= (uint8_t)(((best >> plan.sign_bit[o]) & 1) << o);
    codes[gid] = code;
}

__global__ void from_linear_scales_kernel(ConvertPlan plan, const float *__restrict__ S,
                                          const float *__restrict__ qbias, uint16_t *__restrict__ alpha,
                                          uint16_t *__restrict__ offset, size_t total)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const double s = static_cast<double>(S[gid]);
    for (int o = 0; o < plan.q; ++o) alpha[gid * plan.q + o] = double_to_half_bits(s * plan.alpha_hat[o]);
    // the product is exact in binary64 (24-bit x 9-bit significands), the sum rounds once
    offset[gid] = double_to_half_bits(plan.centre * s + static_cast<double>(qbias[gid]));
}

// Host: validate the tying and derive BCchoice, the plane order (descending alpha_hat) and the
// bit each output plane reads its sign from.  Returns false if a class is empty or a label is bad.
bool make_convert_plan(int n_bits, int q, const int32_t *class_of_plane, ConvertPlan *plan)
{
    if (n_bits < 1 || n_bits > 8 || q < 1 || q > kMaxQ || q > n_bits || !class_of_plane) return false;
    double ah[kMaxQ] = {0, 0, 0, 0};
    int first_bit[kMaxQ] = {-1, -1, -1, -1};
    for (int i = 0; i < n_bits; ++i) {  // plane i+1 of Eq. 9 is bit i, weight 2^(i-1)
        const int c = class_of_plane[i];
        if (c < 0 || c >= q) return false;
        ah[c] += (double)(1 << i) / 2.0;
        if (first_bit[c] < 0) first_bit[c] = i;
    }
    for (int c = 0; c < q; ++c)
        if (first_bit[c] < 0) return false;
    int order[kMaxQ] = {0, 1, 2, 3};
    for (int a = 0; a < q; ++a)  // selection sort, descending; the sums are pairwise different
        for (int b = a + 1; b < q; ++b)
            if (ah[order[b]] > ah[order[a]]) { int t = order[a]; order[a] = order[b]; order[b] = t; }
    plan->n_bits = n_bits; plan->q = q; plan->nchoice = 1 << q;
    plan->centre = ((1 << n_bits) - 1) / 2.0;
    for (int o = 0; o < q; ++o) {
        plan->alpha_hat[o] = ah[order[o]];
        plan->sign_bit[o] = first_bit[order[o]];
    }
    for (int m = 0; m < plan->nchoice; ++m) {  // every sign pattern of the q tied planes
        int v = 0;
        for (int i = 0; i < n_bits; ++i) {
            int o = 0;
            while (order[o] != class_of_plane[i]) ++o;
            if ((m >> o) & 1) v |= 1 << i;
        }
        plan->choice[m] = v;
    }
    for (int a = 0; a < plan->nchoice; ++a)  // ascending
        for (int b = a + 1; b < plan->nchoice; ++b)
            if (plan->choice[b] < plan->choice[a]) { int t = plan->choice[a]; plan->choice[a] = plan->choice[b]; plan->choice[b] = t; }
    return true;
}

hipError_t launch_from_linear(int M, int N, int group, int n_bits, int q, const int32_t *class_of_plane,
                              const uint8_t *w_int, const float *S, const float *qbias, uint8_t *codes,
                              uint16_t *alpha, uint16_t *offset, hipStream_t stream)
{
    ConvertPlan plan;
    if (!make_convert_plan(n_bits, q, class_of_plane, &plan)) return hipErrorInvalidValue;
    const size_t nw = (size_t)M * N, ng = (size_t)M * (N / group);
    hipLaunchKernelGGL(from_linear_codes_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, stream, plan,
                       w_int, codes, nw);
    hipLaunchKernelGGL(from_linear_scales_kernel, dim3((unsigned)((ng + 255) / 256)), dim3(256), 0, stream, plan,
                       S, qbias, alpha, offset, ng);
    return hipGetLastError();
}

}  // namespace bcq
