// Argument checks of the C ABI that need neither a device nor the HIP headers: plain C++, so that a host
// compiler can build them alone (the sanitizer tests do) and bns_api.hip uses the same code.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "../../include/bns.h"

namespace bns {

struct Dims {
    int32_t N, C, H, W;
    int32_t HW;     // H * W
    int32_t dtype;  // bns_dtype
    int32_t vec;    // elements per memory access: largest of {8 (bf16 only), 4, 1} dividing HW
    int32_t layout; // bns_layout
};

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool overlap(const void* a, size_t na, const void* b, size_t nb) {
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

inline bns_status check_shape(const bns_shape* sh, Dims* d) {
    if (!sh) return BNS_EINVAL;
    if (sh->N <= 0 || sh->C <= 0 || sh->H <= 0 || sh->W <= 0) return BNS_EINVAL;
    if (sh->dtype != BNS_F32 && sh->dtype != BNS_BF16) return BNS_EINVAL;
    if (sh->layout != BNS_NCHW && sh->layout != BNS_NHWC) return BNS_EINVAL;
    const int64_t hw = int64_t(sh->H) * sh->W;
    const int64_t lim = int64_t(1) << 31;
    if (sh->N > 65535 || sh->C > (1 << 24) || hw >= lim || hw * sh->N >= lim || hw * sh->C >= lim)
        return BNS_EUNSUPPORTED;
    d->N = sh->N;
    d->C = sh->C;
    d->H = sh->H;
    d->W = sh->W;
    d->HW = int32_t(hw);
    d->dtype = sh->dtype;
    d->layout = sh->layout;
    if (sh->dtype == BNS_BF16 && hw % 8 == 0)
        d->vec = 8;
    else if (hw % 4 == 0)
        d->vec = 4;
    else
        d->vec = 1;
    return BNS_OK;
}

inline bns_status check_spec(const bns_shape* sh, const bns_spec* sp) {
    if (!sp) return BNS_EINVAL;
    switch (sp->mode) {
        case BNS_FULL:
            return BNS_OK;
        case BNS_NS:
        case BNS_BS:
            return (sp->n_s >= 1 && sp->n_s <= sh->N) ? BNS_OK : BNS_EINVAL;   // n_s in (0, N], Alg. 1
        case BNS_VDN:
            return (sp->n_s >= 1 && sp->n_s < sh->N) ? BNS_OK : BNS_EINVAL;    // at least one real sample
        case BNS_FS:
            if (sp->fs_per_channel != 0 && sp->fs_per_channel != 1) return BNS_EINVAL;
            return (sp->patch_h >= 1 && sp->patch_h <= sh->H && sp->patch_w >= 1 && sp->patch_w <= sh->W)
                       ? BNS_OK
                       : BNS_EINVAL;                                           // h_s in (0, H], w_s in (0, W], Alg. 2
        default:
            return BNS_EINVAL;
    }
}

}  // namespace bns
