// Internal helpers shared by the converter (bcq_convert.hip) and the quantiser (bcq_quant.hip):
// how a tying of the n linear bit-planes into q classes (paper Eq. 10) turns into the set of
// representable integers, the plane order and the sign bits of the fused form (Eq. 11), the
// nearest-member rounding of Eq. 6, and the single-rounding binary64 -> binary16 conversion of the
// fused scales.  Not part of the public ABI.
#pragma once
#include <stdint.h>

#include "bcq_layout.h"

namespace bcq {

constexpr int kMaxBits = 8;  // bits of the intermediate linear quantisation

struct TyingPlan {
    int nchoice;              // 2^q
    int choice[16];           // members of BCchoice, ascending
    int sign_bit[kMaxQ];      // output plane o takes its sign from this bit of the rounded integer
    double alpha_hat[kMaxQ];  // sum of 2^(i-2) over the planes i (bits i-1) tied into output plane o; descending
};

// label[i] = class (0..q-1) of bit i, i.e. of plane i+1 of Eq. 9, whose weight is 2^(i-1) = (1 << i) / 2.
// fold = false: a label outside 0..q-1 or an empty class is an error (returns false);
// fold = true:  labels are folded into 0..q-1 and an empty class reads bit 0 (for labels that come
//               from device memory the host cannot inspect).
// Output planes are ordered by descending alpha_hat (the sums are pairwise different: distinct sets
// of powers of two); the sign of plane o is the lowest bit tied into it.
template <class Label>
BCQ_HD inline bool make_tying_plan(int n_bits, int q, const Label *label, bool fold, TyingPlan *plan)
{
    // Every loop has a constant trip count and every array index is a loop counter, so that device code
    // keeps all of this in registers.
    double ah[kMaxQ] = {-1.0, -1.0, -1.0, -1.0};  // classes >= q keep -1 and sort last
    int first_bit[kMaxQ] = {-1, -1, -1, -1};
    int cls[kMaxBits];
    bool ok = true;
    for (int c = 0; c < kMaxQ; ++c)
        if (c < q) ah[c] = 0.0;
    for (int i = 0; i < kMaxBits; ++i) {
        cls[i] = 0;
        if (i < n_bits) {
            int c = (int)label[i];
            if (c < 0 || c >= q) {
                ok = false;
                c = c < 0 ? 0 : q - 1;
            }
            cls[i] = c;
            for (int k = 0; k < kMaxQ; ++k)
                if (k == c) {
                    ah[k] += (double)(1 << i) / 2.0;
                    if (first_bit[k] < 0) first_bit[k] = i;
                }
        }
    }
    for (int c = 0; c < kMaxQ; ++c)
        if (c < q && first_bit[c] < 0) {
            ok = false;
            first_bit[c] = 0;
        }
    if (!ok && !fold) return false;
    // order the classes by descending alpha_hat, carrying their first bit and their index
    int idx[kMaxQ] = {0, 1, 2, 3};
    for (int pass = 0; pass < kMaxQ - 1; ++pass)
        for (int a = 0; a < kMaxQ - 1 - pass; ++a)
            if (ah[a + 1] > ah[a]) {
                const double ta = ah[a]; ah[a] = ah[a + 1]; ah[a + 1] = ta;
                const int tb = first_bit[a]; first_bit[a] = first_bit[a + 1]; first_bit[a + 1] = tb;
                const int ti = idx[a]; idx[a] = idx[a + 1]; idx[a + 1] = ti;
            }
    for (int o = 0; o < kMaxQ; ++o) {
        plan->alpha_hat[o] = o < q ? ah[o] : 0.0;
        plan->sign_bit[o] = o < q ? first_bit[o] : 0;
    }
    plan->nchoice = 1 << q;
    for (int m = 0; m < 16; ++m) {  // every sign pattern of the q classes; unused entries sort last
        int v = 0;
        for (int i = 0; i < kMaxBits; ++i)
            if (i < n_bits && ((m >> cls[i]) & 1)) v |= 1 << i;
        plan->choice[m] = m < plan->nchoice ? v : 0x7fffffff;
    }
    for (int pass = 0; pass < 15; ++pass)  // ascending
        for (int a = 0; a < 15 - pass; ++a)
            if (plan->choice[a + 1] < plan->choice[a]) {
                const int t = plan->choice[a]; plan->choice[a] = plan->choice[a + 1]; plan->choice[a + 1] = t;
            }
    (void)idx;
    return true;
}

// Eq. 6: the member of `choice` (ascending) nearest to w; scanning upwards with a strict
// comparison keeps the smaller member on a tie.
BCQ_HD inline int nearest_choice(int w, const int *choice, int nchoice)
{
    int best = choice[0], best_d = w > choice[0] ? w - choice[0] : choice[0] - w;
    for (int k = 1; k < nchoice; ++k) {
        const int d = w > choice[k] ? w - choice[k] : choice[k] - w;
        if (d < best_d) { best_d = d; best = choice[k]; }
    }
    return best;
}

// Plane code of a member of BCchoice: bit o = sign of fused plane o.
BCQ_HD inline uint8_t code_of(int member, const TyingPlan &plan, int q)
{
    uint8_t code = 0;
    for (int o = 0; o < q; ++o) code |= (uint8_t)(((member >> plan.sign_bit[o]) & 1) << o);
    return code;
}

#if defined(__HIPCC__)
// binary64 -> binary16, round to nearest even, with a single rounding: the value is first
// rounded to binary32 *to odd* (truncate, then set the last bit if anything was lost), which
// keeps enough information for the final rounding to be the correct one.
__device__ __forceinline__ uint16_t double_to_half_bits(double v)
{
    float f = __double2float_rz(v);
    if (static_cast<double>(f) != v && !(v != v)) {
        // |f| <= |v|: set the magnitude's last bit when the truncation lost something (sticky bit)
        f = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, f) | 1u);
    }
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f));
}
#endif

}  // namespace bcq
