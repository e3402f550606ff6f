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
#include "bcq_tying.h"

namespace bcq {

struct ConvertPlan {
    int n_bits, q;
    TyingPlan tying;
    double centre;  // (2^n - 1) / 2
};

__global__ void from_linear_codes_kernel(ConvertPlan plan, const uint8_t *__restrict__ w_int,
                                         uint8_t *__restrict__ codes, size_t total)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int w = w_int[gid] & ((1 << plan.n_bits) - 1);
    codes[gid] = code_of(nearest_choice(w, plan.tying.choice, plan.tying.nchoice), plan.tying, plan.q);  // Eq. 6
}

__global__ void from_linear_scales_kernel(ConvertPlan plan, const float *__restrict__ S,
                                          const float *__restrict__ qbias, uint16_t *__restrict__ alpha,
                                          uint16_t *__restrict__ offset, size_t total)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const double s = static_cast<double>(S[gid]);
    for (int o = 0; o < plan.q; ++o) alpha[gid * plan.q + o] = double_to_half_bits(s * plan.tying.alpha_hat[o]);
    // the product is exact in binary64 (24-bit x 9-bit significands), the sum rounds once
    offset[gid] = double_to_half_bits(plan.centre * s + static_cast<double>(qbias[gid]));
}

// Host: validate the tying and derive BCchoice, the plane order (descending alpha_hat) and the
// bit each output plane reads its sign from.  Returns false if a class is empty or a label is bad.
bool make_convert_plan(int n_bits, int q, const int32_t *class_of_plane, ConvertPlan *plan)
{
    if (n_bits < 1 || n_bits > kMaxBits || q < 1 || q > kMaxQ || q > n_bits || !class_of_plane) return false;
    plan->n_bits = n_bits;
    plan->q = q;
    plan->centre = ((1 << n_bits) - 1) / 2.0;
    return make_tying_plan(n_bits, q, class_of_plane, false, &plan->tying);
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
