// Bad-argument sweep through the real extern "C" entry points of libbns, for a build whose HOST code runs under
// AddressSanitizer and UndefinedBehaviorSanitizer, on a machine without a GPU.  Every call made here has at least
// one invalid argument, so it must come back with the documented status from the host-side validation; the tensor
// addresses are made up and never dereferenced.  The host-only functions (index, sizes, options, strings) are
// called with valid arguments and exactly sized heap buffers.  Exit status 0 and "calls <n>" on success.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <string>
#include <utility>
#include <vector>

#include "../../include/bns.h"

namespace {

enum Field { X, Y, DY, DX, GAMMA, BETA, SM, SI, PARTS, DGAMMA, DBETA, RM, RV, WS, kFields };

struct Args {
    bns_shape shape;
    bns_spec spec;
    int32_t n_v;
    float mix, eps, mom;
    uintptr_t p[kFields];
    size_t wsb;
    bool null_shape, null_spec;
};

enum Entry { FORWARD, BACKWARD, BACKWARD_BUILTIN, STATS, NORMALIZE, REDUCE, DXPASS, FORWARD_MIXED, BACKWARD_MIXED, INFERENCE, kEntries };
const char* kEntryName[kEntries] = {"bns_forward", "bns_backward", "bns_backward_builtin_workspace", "bns_forward_stats",
                                    "bns_forward_normalize", "bns_backward_reduce", "bns_backward_dx", "bns_forward_mixed",
                                    "bns_backward_mixed", "bns_inference"};

struct Uses {
    std::vector<Field> required, aligned;             // non-null pointers; pointers that must be 16-byte aligned
    std::vector<std::pair<Field, Field>> apart;       // tensors that must not overlap
    bool spec, workspace, eps, mom, mixed;
};

const Uses kUses[kEntries] = {
    {{X, GAMMA, BETA, Y, SM, SI, WS}, {X, Y, WS}, {{Y, X}}, true, true, true, true, false},
    {{X, DY, GAMMA, SM, SI, DX, DGAMMA, DBETA, WS}, {X, DY, DX, WS}, {{DX, X}, {DX, DY}}, true, true, false, false, false},
    {{X, DY, GAMMA, SM, SI, DX, DGAMMA, DBETA}, {X, DY, DX}, {{DX, X}, {DX, DY}}, true, false, false, false, false},
    {{X, SM, SI, WS}, {X, WS}, {}, true, true, true, true, false},
    {{X, GAMMA, BETA, SM, SI, Y}, {X, Y}, {{Y, X}}, false, false, false, false, false},
    {{X, DY, SM, SI, DGAMMA, DBETA, WS}, {X, DY, WS}, {}, false, true, false, false, false},
    {{X, DY, GAMMA, SM, SI, DGAMMA, DBETA, DX}, {X, DY, DX}, {{DX, X}, {DX, DY}}, true, false, false, false, false},
    {{X, GAMMA, BETA, Y, SM, SI, PARTS, WS}, {X, Y, WS}, {{Y, X}}, true, true, true, true, true},
    {{X, DY, GAMMA, SM, SI, PARTS, DX, DGAMMA, DBETA, WS}, {X, DY, DX, WS}, {{DX, X}, {DX, DY}}, true, true, false, false, true},
    {{X, GAMMA, BETA, RM, RV, Y}, {X, Y}, {{Y, X}}, false, false, true, false, false},
};

template <typename T>
T* ptr(const Args& a, Field f) {
    return reinterpret_cast<T*>(a.p[f]);
}

bns_status call(Entry e, const Args& a) {
    const bns_shape* sh = a.null_shape ? nullptr : &a.shape;
    const bns_spec* sp = a.null_spec ? nullptr : &a.spec;
    switch (e) {
        case FORWARD:
            return bns_forward(sh, sp, 1, ptr<void>(a, X), ptr<float>(a, GAMMA), ptr<float>(a, BETA), a.eps, a.mom,
                               ptr<void>(a, Y), ptr<float>(a, SM), ptr<float>(a, SI), ptr<float>(a, RM), ptr<float>(a, RV),
                               ptr<void>(a, WS), a.wsb, nullptr);
        case BACKWARD:
            return bns_backward(sh, sp, 1, ptr<void>(a, X), ptr<void>(a, DY), ptr<float>(a, GAMMA), ptr<float>(a, SM),
                                ptr<float>(a, SI), ptr<void>(a, DX), ptr<float>(a, DGAMMA), ptr<float>(a, DBETA),
                                ptr<void>(a, WS), a.wsb, nullptr);
        case BACKWARD_BUILTIN:
            return bns_backward_builtin_workspace(sh, sp, 1, ptr<void>(a, X), ptr<void>(a, DY), ptr<float>(a, GAMMA),
                                                  ptr<float>(a, SM), ptr<float>(a, SI), ptr<void>(a, DX),
                                                  ptr<float>(a, DGAMMA), ptr<float>(a, DBETA), nullptr);
        case STATS:
            return bns_forward_stats(sh, sp, 1, ptr<void>(a, X), a.eps, a.mom, ptr<float>(a, SM), ptr<float>(a, SI),
                                     ptr<float>(a, RM), ptr<float>(a, RV), ptr<void>(a, WS), a.wsb, nullptr);
        case NORMALIZE:
            return bns_forward_normalize(sh, ptr<void>(a, X), ptr<float>(a, GAMMA), ptr<float>(a, BETA), ptr<float>(a, SM),
                                         ptr<float>(a, SI), ptr<void>(a, Y), nullptr);
        case REDUCE:
            return bns_backward_reduce(sh, ptr<void>(a, X), ptr<void>(a, DY), ptr<float>(a, SM), ptr<float>(a, SI),
                                       ptr<float>(a, DGAMMA), ptr<float>(a, DBETA), ptr<void>(a, WS), a.wsb, nullptr);
        case DXPASS:
            return bns_backward_dx(sh, sp, 1, ptr<void>(a, X), ptr<void>(a, DY), ptr<float>(a, GAMMA), ptr<float>(a, SM),
                                   ptr<float>(a, SI), ptr<float>(a, DGAMMA), ptr<float>(a, DBETA), ptr<void>(a, DX), nullptr);
        case FORWARD_MIXED:
            return bns_forward_mixed(sh, sp, 1, a.n_v, a.mix, ptr<void>(a, X), ptr<float>(a, GAMMA), ptr<float>(a, BETA),
                                     a.eps, a.mom, ptr<void>(a, Y), ptr<float>(a, SM), ptr<float>(a, SI),
                                     ptr<float>(a, PARTS), ptr<float>(a, RM), ptr<float>(a, RV), ptr<void>(a, WS), a.wsb,
                                     nullptr);
        case BACKWARD_MIXED:
            return bns_backward_mixed(sh, sp, 1, a.n_v, a.mix, ptr<void>(a, X), ptr<void>(a, DY), ptr<float>(a, GAMMA),
                                      ptr<float>(a, SM), ptr<float>(a, SI), ptr<float>(a, PARTS), ptr<void>(a, DX),
                                      ptr<float>(a, DGAMMA), ptr<float>(a, DBETA), ptr<void>(a, WS), a.wsb, nullptr);
        case INFERENCE:
            return bns_inference(sh, ptr<void>(a, X), ptr<float>(a, GAMMA), ptr<float>(a, BETA), ptr<float>(a, RM),
                                 ptr<float>(a, RV), a.eps, ptr<void>(a, Y), nullptr);
        default:
            return BNS_OK;
    }
}

size_t g_calls = 0;
int g_failures = 0;

void expect(Entry e, const Args& a, bns_status want, bns_status also, const char* what) {
    const bns_status got = call(e, a);
    ++g_calls;
    if (got != want && got != also) {
        fprintf(stderr, "%s, %s: status %d (%s), expected %d\n", kEntryName[e], what, int(got), bns_status_string(got),
                int(want));
        ++g_failures;
    }
}

Args valid_args(int32_t layout, int32_t dtype) {
    Args a;
    memset(&a, 0, sizeof a);
    a.shape = bns_shape{8, 4, 6, 6, dtype, layout};
    a.spec.mode = BNS_BS;
    a.spec.n_s = 2;
    a.spec.patch_h = a.spec.patch_w = 3;
    a.n_v = 2;
    a.mix = 0.5f, a.eps = 1e-5f, a.mom = 0.1f;
    for (int f = 0; f < kFields; ++f) a.p[f] = uintptr_t(0x100000) * uintptr_t(f + 1);     // far apart, 16-byte aligned
    a.wsb = bns_workspace_bytes(&a.shape, &a.spec);
    return a;
}

void sweep_entry(Entry e, int32_t layout, int32_t dtype) {
    const Uses& u = kUses[e];
    const Args ok = valid_args(layout, dtype);
    const size_t tensor_bytes = size_t(8) * 4 * 36 * (dtype == BNS_F32 ? 4 : 2);
    Args a = ok;
    a.null_shape = true;
    expect(e, a, BNS_EINVAL, BNS_EINVAL, "null shape");
    if (u.spec) {
        a = ok;
        a.null_spec = true;
        expect(e, a, BNS_EINVAL, BNS_EINVAL, "null spec");
    }
    for (Field f : u.required) {
        a = ok;
        a.p[f] = 0;
        expect(e, a, BNS_EINVAL, BNS_EINVAL, "null pointer");
    }
    for (Field f : u.aligned)
        for (uintptr_t off : {1u, 2u, 4u, 8u, 15u}) {
            a = ok;
            a.p[f] += off;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "misaligned pointer");
        }
    for (const auto& pr : u.apart)
        for (size_t off : {size_t(0), size_t(16), tensor_bytes - 16}) {
            a = ok;
            a.p[pr.first] = a.p[pr.second] + off;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "output over input");
            a = ok;
            a.p[pr.second] = a.p[pr.first] + off;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "input over output");
        }
    if (u.workspace)
        for (size_t wsb : {size_t(0), size_t(1), size_t(255), size_t(256), ok.wsb - 1}) {
            a = ok;
            a.wsb = wsb;
            expect(e, a, BNS_EWORKSPACE, BNS_EWORKSPACE, "small workspace");
        }
    if (u.eps)
        for (float eps : {-1.f, -0.f - 1e-30f, float(NAN), -float(INFINITY)}) {
            a = ok;
            a.eps = eps;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "eps");
        }
    if (u.mom)
        for (float mom : {-0.5f, 1.5f, float(NAN), float(INFINITY)}) {
            a = ok;
            a.mom = mom;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "momentum");
        }
    if (u.mixed) {
        for (float mix : {-0.1f, 1.1f, float(NAN)}) {
            a = ok;
            a.mix = mix;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "mix_beta");
        }
        for (int32_t n_v : {INT32_MIN, -1, 0, 7, 8, 9, INT32_MAX}) {       // 7: n_s = 2 exceeds the one real sample
            a = ok;
            a.n_v = n_v;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "n_v");
        }
        a = ok;
        a.spec.mode = BNS_VDN;
        expect(e, a, BNS_EINVAL, BNS_EINVAL, "VDN inside VDN + sampling");
    }
    // extents and enums
    const int32_t ext[] = {INT32_MIN, -1, 0, INT32_MAX};
    for (int k = 0; k < 4; ++k)
        for (int32_t v : ext) {
            a = ok;
            (&a.shape.N)[k] = v;
            expect(e, a, BNS_EINVAL, BNS_EUNSUPPORTED, "extent");
        }
    a = ok;
    a.shape.N = 65536;
    expect(e, a, BNS_EUNSUPPORTED, BNS_EUNSUPPORTED, "N beyond the limit");
    a = ok;
    a.shape.C = (1 << 24) + 1;
    expect(e, a, BNS_EUNSUPPORTED, BNS_EUNSUPPORTED, "C beyond the limit");
    a = ok;
    a.shape.H = a.shape.W = 50000;
    expect(e, a, BNS_EUNSUPPORTED, BNS_EUNSUPPORTED, "H * W");
    for (int32_t v : {INT32_MIN, -1, 2, 77, INT32_MAX}) {
        a = ok;
        a.shape.dtype = v;
        expect(e, a, BNS_EINVAL, BNS_EINVAL, "dtype");
        a = ok;
        a.shape.layout = v;
        expect(e, a, BNS_EINVAL, BNS_EINVAL, "layout");
    }
    if (u.spec) {
        for (int32_t v : {INT32_MIN, -1, 5, INT32_MAX}) {
            a = ok;
            a.spec.mode = v;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "mode");
        }
        for (int32_t mode : {int32_t(BNS_NS), int32_t(BNS_BS)})
            for (int32_t v : {INT32_MIN, -1, 0, 9, INT32_MAX}) {
                a = ok;
                a.spec.mode = mode;
                a.spec.n_s = v;
                expect(e, a, BNS_EINVAL, BNS_EINVAL, "n_s");
            }
        if (!u.mixed)
            for (int32_t v : {INT32_MIN, 0, 8, INT32_MAX}) {
                a = ok;
                a.spec.mode = BNS_VDN;
                a.spec.n_s = v;
                expect(e, a, BNS_EINVAL, BNS_EINVAL, "VDN n_s");
            }
        for (int32_t v : {INT32_MIN, -1, 0, 7, INT32_MAX}) {
            a = ok;
            a.spec.mode = BNS_FS;
            a.spec.patch_h = v;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "patch_h");
            a = ok;
            a.spec.mode = BNS_FS;
            a.spec.patch_w = v;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "patch_w");
        }
        for (int32_t v : {INT32_MIN, -1, 2, INT32_MAX}) {
            a = ok;
            a.spec.mode = BNS_FS;
            a.spec.fs_per_channel = v;
            expect(e, a, BNS_EINVAL, BNS_EINVAL, "fs_per_channel");
        }
        if (layout == BNS_NHWC && e != BACKWARD_BUILTIN) {
            a = ok;
            a.spec.mode = BNS_FS;
            a.spec.fs_per_channel = 1;
            a.wsb = size_t(1) << 30;
            expect(e, a, BNS_EUNSUPPORTED, BNS_EUNSUPPORTED, "per-channel patches in N x H x W x C");
        }
    }
}

void host_functions() {
    // exactly sized heap buffers: a write past C boxes is an AddressSanitizer report
    for (int32_t C : {1, 3, 257})
        for (int32_t mode = BNS_FULL; mode <= BNS_VDN; ++mode)
            for (int32_t pc = 0; pc < 2; ++pc) {
                bns_shape sh = {9, C, 11, 13, BNS_BF16, pc ? BNS_NCHW : BNS_NHWC};
                bns_spec sp;
                memset(&sp, 0, sizeof sp);
                sp.mode = mode, sp.n_s = 4, sp.patch_h = 5, sp.patch_w = 13, sp.fs_per_channel = pc;
                sp.layer_id = 0xFFFFFFFFu, sp.epoch = 0xFFFFFFFFu;
                std::vector<bns_box> boxes(static_cast<size_t>(C));
                ++g_calls;
                if (bns_sample_index(&sh, &sp, ~uint64_t(0), boxes.data()) != BNS_OK) ++g_failures, fprintf(stderr, "index\n");
                if (mode != BNS_VDN) {
                    ++g_calls;
                    if (bns_sample_index_mixed(&sh, &sp, 5, 3, boxes.data()) != BNS_OK) ++g_failures, fprintf(stderr, "mixed index\n");
                    for (const bns_box& b : boxes)
                        if (b.n0 < 3 || b.n0 + b.n_cnt > 9) ++g_failures, fprintf(stderr, "mixed box outside the real samples\n");
                }
                if (bns_sample_index(&sh, &sp, 0, nullptr) != BNS_EINVAL) ++g_failures;
                if (bns_sample_index_device(&sh, &sp, 0, nullptr, nullptr) != BNS_EINVAL) ++g_failures;
                if (bns_workspace_bytes(&sh, &sp) < 256) ++g_failures, fprintf(stderr, "workspace size\n");
            }
    if (bns_workspace_bytes(nullptr, nullptr) != 0) ++g_failures;
    bns_shape big = {65535, 1, 181, 181, BNS_F32, BNS_NCHW};          // N*H*W just below 2^31
    if (bns_workspace_bytes(&big, nullptr) == 0) ++g_failures, fprintf(stderr, "largest N\n");
    bns_shape wide = {2, 1 << 24, 1, 1, BNS_F32, BNS_NHWC};
    if (bns_workspace_bytes(&wide, nullptr) < (size_t(1) << 24) * 8) ++g_failures, fprintf(stderr, "largest C\n");
    for (int s = 0; s < 8; ++s)                                  // 5..7: no such status, still a string
        if (!bns_status_string(bns_status(s)) || !bns_status_string(bns_status(s))[0]) ++g_failures;
    if (bns_moving_average_weight(0, 0.3f) != 1.f || bns_moving_average_weight(1, 0.3f) != 1.f ||
        bns_moving_average_weight(2, 0.3f) != 0.3f || bns_moving_average_weight(~uint64_t(0), 0.3f) != 0.3f)
        ++g_failures, fprintf(stderr, "moving-average weight\n");
    // options: unknown, missing and oversized names, values at and beyond the ends
    const std::string longname(100000, 'x');
    if (bns_set_option(nullptr, 1) != BNS_EINVAL || bns_set_option("", 1) != BNS_EINVAL ||
        bns_set_option(longname.c_str(), 1) != BNS_EINVAL || bns_get_option(nullptr) != -1 ||
        bns_get_option(longname.c_str()) != -1 || bns_set_option("path", -1) != BNS_EINVAL ||
        bns_set_option("path", INT32_MAX) != BNS_EINVAL || bns_set_option("path", INT32_MIN) != BNS_EINVAL)
        ++g_failures, fprintf(stderr, "options\n");
    const char* names[] = {"path", "fused_variant", "fused_pipe", "fused_team", "fused_coop", "fused_keep_x", "fused_patch_mask", "split_statistics",
                           "splits_stats", "splits_reduce", "channel_group", "nhwc_blocks", "nhwc_ew_rows", "nhwc_small", "nhwc_split_dx",
                           "norm_unroll", "dx_unroll", "reduce_unroll", "norm_nt", "dx_nt", "reduce_nt", "cache_reuse", "test_spin_limit",
                           "test_mute_exchange"};
    for (const char* n : names) {
        if (bns_get_option(n) != 0) ++g_failures, fprintf(stderr, "option %s not at its default\n", n);
        if (bns_set_option(n, 1) != BNS_OK || bns_get_option(n) != 1) ++g_failures, fprintf(stderr, "option %s\n", n);
        bns_set_option(n, INT32_MAX);                                  // accepted only by channel_group
        if (bns_set_option(n, 0) != BNS_OK || bns_get_option(n) != 0) ++g_failures, fprintf(stderr, "option %s reset\n", n);
        ++g_calls;
    }
    int32_t out = 7;
    if (bns_expired_waits(reinterpret_cast<void*>(0x10000), 4096, nullptr, nullptr) != BNS_EINVAL ||
        bns_expired_waits(reinterpret_cast<void*>(0x10004), 4096, nullptr, &out) != BNS_EINVAL ||
        bns_expired_waits(reinterpret_cast<void*>(0x10000), 255, nullptr, &out) != BNS_EWORKSPACE || out != 7)
        ++g_failures, fprintf(stderr, "bns_expired_waits\n");
    void* const a = reinterpret_cast<void*>(0x10000);
    void* const b = reinterpret_cast<void*>(0x20000);
    if (bns_copy_reference(a, b, 60, nullptr) != BNS_EINVAL || bns_copy_reference(a, reinterpret_cast<void*>(0x10020), 64, nullptr) != BNS_EINVAL ||
        bns_copy_reference(nullptr, b, 64, nullptr) != BNS_EINVAL || bns_copy_reference(a, nullptr, 64, nullptr) != BNS_EINVAL ||
        bns_copy_reference(a, reinterpret_cast<void*>(0x20008), 64, nullptr) != BNS_EINVAL)
        ++g_failures, fprintf(stderr, "bns_copy_reference\n");
}

}  // namespace

int main() {
    for (int e = 0; e < kEntries; ++e)
        for (int32_t layout : {int32_t(BNS_NCHW), int32_t(BNS_NHWC)})
            for (int32_t dtype : {int32_t(BNS_F32), int32_t(BNS_BF16)}) sweep_entry(Entry(e), layout, dtype);
    host_functions();
    printf("calls %zu failures %d\n", g_calls, g_failures);
    return g_failures ? 1 : 0;
}
