// C ABI of libbns: argument validation and launch sequencing.  See include/bns.h for
// the contract of every entry point.  No allocation, no synchronisation, no state
// except the tuning overrides.
#include <hip/hip_runtime.h>
#include <string.h>

#include <atomic>

#include "../../include/bns.h"
#include "bns_internal.hpp"

using namespace bns;

std::atomic<uint32_t> bns::g_launch_count{0};
thread_local int32_t bns::t_last_fused_backward = 0;
thread_local int32_t bns::t_last_fused_forward = 0;

// Built-in scratch memory of bns_backward_builtin_workspace (see there).
constexpr size_t kBuiltinWorkspaceBytes = (size_t(4) << 20) + bns::kHeaderBytes;    // 3840 channels
static __device__ __align__(256) unsigned char scratch[kBuiltinWorkspaceBytes];

namespace {

std::atomic<int32_t> g_splits_stats{0};
std::atomic<int32_t> g_splits_reduce{0};
std::atomic<int32_t> g_channel_group{0};
// What the calling thread's last forward / backward call launched: 1 = streaming kernels,
// 2 = fused single-launch kernel, 3 = one-launch kernel for small N x H x W x C tensors, 4 = streaming kernels with dx
// split between the reduction kernel (rows outside S) and a kernel for the rows of S (N x H x W x C).
thread_local int32_t t_last_path_forward = 0;
thread_local int32_t t_last_path_backward = 0;

inline size_t elem_bytes(const Dims& d) { return d.dtype == BNS_F32 ? 4 : 2; }
inline size_t tensor_bytes(const Dims& d) { return size_t(d.N) * d.C * d.HW * elem_bytes(d); }
inline size_t partial_bytes(const Dims& d) { return (size_t(d.C) * kMaxSplits * sizeof(Partial) + 255) & ~size_t(255); }
inline bool nhwc(const Dims& d) { return d.layout == BNS_NHWC; }
// Workspace layout: [header][sums S][sums V][slots] (N x H x W x C: no slots).  The header comes first so that
// bns_expired_waits finds it without knowing the shape.
inline size_t workspace_need(const Dims& d) {
    if (nhwc(d)) return kHeaderBytes + 2 * nhwc_partial_bytes(d);
    return kHeaderBytes + 2 * partial_bytes(d) + kSlotBytes;
}
inline Partial* partials_of(void* workspace) {
    return reinterpret_cast<Partial*>(static_cast<char*>(workspace) + kHeaderBytes);
}
inline void* slots_of(void* workspace, const Dims& d) {
    return static_cast<char*>(workspace) + kHeaderBytes + 2 * partial_bytes(d);
}
// N x H x W x C: one location set for all channels
inline bns_status check_layout(const Dims& d, const bns_spec* sp) {
    return (nhwc(d) && sp->mode == BNS_FS && sp->fs_per_channel) ? BNS_EUNSUPPORTED : BNS_OK;
}

inline bns_status dev(hipError_t e) { return e == hipSuccess ? BNS_OK : BNS_EDEVICE; }

// Launch-choice overrides reachable through bns_set_option / bns_get_option.  Value 0 = automatic;
// non-temporal masks are given as mask + 1 so that 0 keeps that meaning.
struct TuningEntry {
    const char* name;
    TuneInt Tuning::*field;
    int hi, bias;
    bool pow2;      // unroll factors: 1, 2 or 4
};
const TuningEntry kTuningTable[] = {
    {"norm_unroll", &Tuning::norm_unroll, 4, 0, true},     {"norm_nt", &Tuning::norm_nt, 4, 1, false},
    {"dx_unroll", &Tuning::dx_unroll, 4, 0, true},         {"dx_nt", &Tuning::dx_nt, 4, 1, false},
    {"reduce_unroll", &Tuning::reduce_unroll, 4, 0, true}, {"reduce_nt", &Tuning::reduce_nt, 4, 1, false},
    {"path", &Tuning::path, 2, 0, false},
    {"fused_variant", &Tuning::fused_variant, 7, 0, false},
    {"fused_pipe", &Tuning::fused_pipe, 16, 0, false},
    {"fused_team", &Tuning::fused_team, 128, 0, false},
    {"fused_coop", &Tuning::fused_coop, 1, 0, false},
    {"test_spin_limit", &Tuning::test_spin_limit, 1 << 21, 0, false},
    {"test_mute_exchange", &Tuning::test_mute_exchange, 1, 0, false},
    {"fused_keep_x", &Tuning::fused_keep_x, 2, 0, false},
    {"fused_patch_mask", &Tuning::fused_patch_mask, 2, 0, false},
    {"split_statistics", &Tuning::split_statistics, 1, 0, false},
    {"nhwc_blocks", &Tuning::nhwc_blocks, kNhwcBlocksMax, 0, false},
    {"nhwc_ew_rows", &Tuning::nhwc_ew_rows, 1 << 20, 0, false},
    {"nhwc_small", &Tuning::nhwc_small, 2, 0, false},
    {"nhwc_split_dx", &Tuning::nhwc_split_dx, 2, 0, false},
    {"cache_reuse", &Tuning::cache_reuse, 2, 0, false},
};

int stats_splits(const Dims& d, const IndexParams& ip, int cg) {
    const int32_t o = g_splits_stats.load();
    if (o > 0) return o;
    const bns_box& b = ip.shared;
    const bool planes = !ip.per_channel && b.h_cnt == d.H && b.w_cnt == d.W && d.vec > 1;
    const uint64_t pts = uint64_t(b.n_cnt) * b.h_cnt * b.w_cnt;
    return auto_splits(cg, uint32_t(planes ? pts / d.vec : pts / 4));
}

int reduce_splits(const Dims& d, int cg) {
    const int32_t o = g_splits_reduce.load();
    if (o > 0) return o;
    return auto_splits(cg, uint32_t(uint64_t(d.N) * d.HW / d.vec));
}

int channel_group(const Dims& d) {
    const int32_t o = g_channel_group.load();
    if (o > 0 && o < d.C) return o;
    return d.C;
}

// ---- stage bodies on a channel range (arguments already validated) ----------------
bns_status stats_range(const Dims& d, const IndexParams& ip, const void* x, float eps, float momentum,
                       float* save_mean, float* save_invstd, float* rm, float* rv, Partial* ws, int c0, int cg,
                       hipStream_t st) {
    if (!g_tuning.split_statistics && g_splits_stats.load() == 0) {
        hipError_t e = hipSuccess;
        if (launch_stats_one_block(d, ip, x, c0, cg, eps, momentum, save_mean, save_invstd, rm, rv, st, &e)) return dev(e);
    }
    const int splits = stats_splits(d, ip, cg);
    if (launch_stats_partial(d, ip, x, ws, splits, c0, cg, st) != hipSuccess) return BNS_EDEVICE;
    return dev(launch_stats_finalize(d, ip, x, ws, splits, c0, cg, eps, momentum, save_mean, save_invstd, rm, rv, st));
}

bns_status reduce_range(const Dims& d, const void* x, const void* dy, const float* save_mean,
                        const float* save_invstd, float* dgamma, float* dbeta, Partial* ws, int c0, int cg,
                        bool x_again, hipStream_t st) {
    const int splits = reduce_splits(d, cg);
    if (launch_reduce_partial(d, x, dy, save_mean, ws, splits, c0, cg, x_again, st) != hipSuccess) return BNS_EDEVICE;
    return dev(launch_reduce_finalize(d, ws, splits, c0, cg, save_invstd, dgamma, dbeta, st));
}

}  // namespace

extern "C" {

const char* bns_status_string(bns_status s) {
    switch (s) {
        case BNS_OK: return "BNS_OK";
        case BNS_EINVAL: return "BNS_EINVAL: invalid argument";
        case BNS_EUNSUPPORTED: return "BNS_EUNSUPPORTED: extent beyond the supported limits";
        case BNS_EWORKSPACE: return "BNS_EWORKSPACE: workspace too small";
        case BNS_EDEVICE: return "BNS_EDEVICE: HIP launch failed";
        default: return "unknown bns_status";
    }
}

bns_status bns_sample_index(const bns_shape* shape, const bns_spec* spec, uint64_t seed, bns_box* boxes) {
    Dims d;
    bns_status s = check_shape(shape, &d);
    if (s != BNS_OK) return s;
    if ((s = check_spec(shape, spec)) != BNS_OK) return s;
    if (!boxes) return BNS_EINVAL;
    const IndexParams ip = make_index_params(*shape, *spec, seed);
    for (int c = 0; c < d.C; ++c) boxes[c] = box_of_channel(ip, c);
    return BNS_OK;
}

bns_status bns_sample_index_device(const bns_shape* shape, const bns_spec* spec, uint64_t seed, bns_box* boxes,
                                   void* stream) {
    Dims d;
    bns_status s = check_shape(shape, &d);
    if (s != BNS_OK) return s;
    if ((s = check_spec(shape, spec)) != BNS_OK) return s;
    if (!boxes) return BNS_EINVAL;
    const IndexParams ip = make_index_params(*shape, *spec, seed);
    return dev(launch_index_boxes(ip, d.C, boxes, static_cast<hipStream_t>(stream)));
}

size_t bns_workspace_bytes(const bns_shape* shape, const bns_spec* spec) {
    (void)spec;
    Dims d;
    if (check_shape(shape, &d) != BNS_OK) return 0;
    return workspace_need(d);
}

bns_status bns_forward_stats(const bns_shape* shape, const bns_spec* spec, uint64_t seed, const void* x, float eps,
                             float momentum, float* save_mean, float* save_invstd, float* running_mean,
                             float* running_var, void* workspace, size_t workspace_bytes, void* stream) {
    Dims d;
    bns_status s = check_shape(shape, &d);
    if (s != BNS_OK) return s;
    if ((s = check_spec(shape, spec)) != BNS_OK) return s;
    if (!x || !save_mean || !save_invstd || !workspace) return BNS_EINVAL;
    if (!aligned16(x) || !aligned16(workspace)) return BNS_EINVAL;
    if (!(eps >= 0.f) || !(momentum >= 0.f && momentum <= 1.f)) return BNS_EINVAL;
    if ((s = check_layout(d, spec)) != BNS_OK) return s;
    if (workspace_bytes < workspace_need(d)) return BNS_EWORKSPACE;
    const IndexParams ip = make_index_params(*shape, *spec, seed);
    if (nhwc(d))
        return dev(launch_nhwc_stats(d, ip.shared, x, partials_of(workspace), eps, momentum, save_mean,
                                     save_invstd, running_mean, running_var, static_cast<hipStream_t>(stream)));
    return stats_range(d, ip, x, eps, momentum, save_mean, save_invstd, running_mean, running_var,
                       partials_of(workspace), 0, d.C, static_cast<hipStream_t>(stream));
}

bns_status bns_forward_normalize(const bns_shape* shape, const void* x, const float* gamma, const float* beta,
                                 const float* save_mean, const float* save_invstd, void* y, void* stream) {
    Dims d;
    bns_status s = check_shape(shape, &d);
    if (s != BNS_OK) return s;
    if (!x || !gamma || !beta || !save_mean || !save_invstd || !y) return BNS_EINVAL;
    if (!aligned16(x) || !aligned16(y)) return BNS_EINVAL;
    if (overlap(x, tensor_bytes(d), y, tensor_bytes(d))) return BNS_EINVAL;
    if (nhwc(d))
        return dev(launch_nhwc_normalize(d, x, gamma, beta, save_mean, save_invstd, y, static_cast<hipStream_t>(stream)));
    return dev(launch_normalize(d, x, gamma, beta, save_mean, save_invstd, y, 0, d.C, static_cast<hipStream_t>(stream)));
}

bns_status bns_inference(const bns_shape* shape, const void* x, const float* gamma, const float* beta,
                         const float* running_mean, const float* running_var, float eps, void* y, void* stream) {
    Dims d;
    bns_status s = check_shape(shape, &d);
    if (s != BNS_OK) return s;
    if (!x || !gamma || !beta || !running_mean || !running_var || !y) return BNS_EINVAL;
    if (!aligned16(x) || !aligned16(y)) return BNS_EINVAL;
    if (!(eps >= 0.f)) return BNS_EINVAL;
    if (overlap(x, tensor_bytes(d), y, tensor_bytes(d))) return BNS_EINVAL;
    if (nhwc(d))
        return dev(launch_nhwc_normalize(d, x, gamma, beta, running_mean, running_var, y,
                                         static_cast<hipStream_t>(stream), eps));
    return dev(launch_normalize(d, x, gamma, beta, running_mean, running_var, y, 0, d.C,
                                static_cast<hipStream_t>(stream), eps));
}

bns_status bns_forward(const bns_shape* shape, const bns_spec* spec, uint64_t seed, const void* x,
                       const float* gamma, const float* beta, float eps, float momentum, void* y, float* save_mean,
                       float* save_invstd, float* running_mean, float* running_var, void* workspace,
                       size_t workspace_bytes, void* stream) {
    Dims d;
    bns_status s = check_shape(shape, &d);
    if (s != BNS_OK) return s;
    if ((s = check_spec(shape, spec)) != BNS_OK) return s;
    if (!x || !gamma || !beta || !y || !save_mean || !save_invstd || !workspace) return BNS_EINVAL;
    if (!aligned16(x) || !aligned16(y) || !aligned16(workspace)) return BNS_EINVAL;
    if (overlap(x, tensor_bytes(d), y, tensor_bytes(d))) return BNS_EINVAL;
    if (!(eps >= 0.f) || !(momentum >= 0.f && momentum <= 1.f)) return BNS_EINVAL;
    if ((s = check_layout(d, spec)) != BNS_OK) return s;
    if (workspace_bytes < workspace_need(d)) return BNS_EWORKSPACE;
    const IndexParams ip = make_index_params(*shape, *spec, seed);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Partial* ws = partials_of(workspace);
    if (nhwc(d)) {
        if (g_tuning.path == 2) return BNS_EUNSUPPORTED;
        hipError_t se = hipSuccess;
        if (launch_nhwc_small_forward(d, ip.shared, x, gamma, beta, eps, momentum, y, save_mean, save_invstd, running_mean,
                                      running_var, st, &se)) {
            t_last_path_forward = 3;
            return dev(se);
        }
        t_last_path_forward = 1;
        if (launch_nhwc_stats(d, ip.shared, x, ws, eps, momentum, save_mean, save_invstd, running_mean, running_var,
                              st) != hipSuccess)
            return BNS_EDEVICE;
        return dev(launch_nhwc_normalize(d, x, gamma, beta, save_mean, save_invstd, y, st));
    }
    if (g_tuning.path != 1) {
        FusedIo io;
        io.x = x;
        io.out = y;
        io.gamma = gamma;
        io.beta = beta;
        io.save_mean = save_mean;
        io.save_invstd = save_invstd;
        io.running_mean = running_mean;
        io.running_var = running_var;
        const hipError_t fe = launch_fused(d, ip, false, io, eps, momentum,
                                           workspace, slots_of(workspace, d), kSlotBytes, 0, d.C, st);
        if (fe == hipSuccess) {
            t_last_path_forward = 2;
            return BNS_OK;
        }
        if (fe != hipErrorNotSupported) return BNS_EDEVICE;
        if (g_tuning.path == 2) return BNS_EUNSUPPORTED;
    }
    t_last_path_forward = 1;
    const int G = channel_group(d);
    for (int c0 = 0; c0 < d.C; c0 += G) {
        const int cg = (d.C - c0 < G) ? d.C - c0 : G;
        s = stats_range(d, ip, x, eps, momentum, save_mean, save_invstd, running_mean, running_var, ws, c0, cg, st);
        if (s != BNS_OK) return s;
        s = dev(launch_normalize(d, x, gamma, beta, save_mean, save_invstd, y, c0, cg, st));
        if (s != BNS_OK) return s;
    }
    return BNS_OK;
}

bns_status bns_backward_reduce(const bns_shape* shape, const void* x, const void* dy, const float* save_mean,
                               const float* save_invstd, float* dgamma, float* dbeta, void* workspace,
                               size_t workspace_bytes, void* stream) {
    Dims d;
    bns_status s = check_shape(shape, &d);
    if (s != BNS_OK) return s;
    if (!x || !dy || !save_mean || !save_invstd || !dgamma || !dbeta || !workspace) return BNS_EINVAL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(workspace)) return BNS_EINVAL;
    if (workspace_bytes < workspace_need(d)) return BNS_EWORKSPACE;
    if (nhwc(d))
        return dev(launch_nhwc_reduce(d, x, dy, save_mean, save_invstd, partials_of(workspace), dgamma, dbeta, false,
                                      static_cast<hipStream_t>(stream)));
    // (the location set is not known here: dy is taken to be what the dx pass reads again)
    return reduce_range(d, x, dy, save_mean, save_invstd, dgamma, dbeta, partials_of(workspace), 0, d.C, false,
                        static_cast<hipStream_t>(stream));
}

bns_status bns_backward_dx(const bns_shape* shape, const bns_spec* spec, uint64_t seed, const void* x,
                           const void* dy, const float* gamma, const float* save_mean, const float* save_invstd,
                           const float* dgamma, const float* dbeta, void* dx, void* stream) {
    Dims d;
    bns_status s = check_shape(shape, &d);
    if (s != BNS_OK) return s;
    if ((s = check_spec(shape, spec)) != BNS_OK) return s;
    if (!x || !dy || !gamma || !save_mean || !save_invstd || !dgamma || !dbeta || !dx) return BNS_EINVAL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx)) return BNS_EINVAL;
    const size_t tb = tensor_bytes(d);
    if (overlap(dx, tb, x, tb) || overlap(dx, tb, dy, tb)) return BNS_EINVAL;
    if ((s = check_layout(d, spec)) != BNS_OK) return s;
    const IndexParams ip = make_index_params(*shape, *spec, seed);
    if (nhwc(d))
        return dev(launch_nhwc_dx(d, ip.shared, x, dy, gamma, save_mean, save_invstd, dgamma, dbeta, dx,
                                  static_cast<hipStream_t>(stream)));
    return dev(launch_dx(d, ip, x, dy, gamma, save_mean, save_invstd, dgamma, dbeta, dx, 0, d.C,
                         static_cast<hipStream_t>(stream)));
}

namespace {
// Host-side checks of bns_backward's tensor arguments (everything but the workspace); fills `d`.
bns_status backward_check(const bns_shape* shape, const bns_spec* spec, const void* x, const void* dy,
                          const float* gamma, const float* save_mean, const float* save_invstd, const void* dx,
                          const float* dgamma, const float* dbeta, Dims* dims) {
    Dims& d = *dims;
    bns_status s = check_shape(shape, &d);
    if (s != BNS_OK) return s;
    if ((s = check_spec(shape, spec)) != BNS_OK) return s;
    if (!x || !dy || !gamma || !save_mean || !save_invstd || !dx || !dgamma || !dbeta) return BNS_EINVAL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx)) return BNS_EINVAL;
    const size_t tb = tensor_bytes(d);
    if (overlap(dx, tb, x, tb) || overlap(dx, tb, dy, tb)) return BNS_EINVAL;
    return check_layout(d, spec);
}

bns_status backward_impl(const bns_shape* shape, const bns_spec* spec, uint64_t seed, const void* x, const void* dy,
                         const float* gamma, const float* save_mean, const float* save_invstd, void* dx,
                         float* dgamma, float* dbeta, void* workspace, size_t workspace_bytes, void* stream,
                         bool order_streams) {
    Dims d;
    bns_status s = backward_check(shape, spec, x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta, &d);
    if (s != BNS_OK) return s;
    if (!workspace || !aligned16(workspace)) return BNS_EINVAL;
    if (workspace_bytes < workspace_need(d)) return BNS_EWORKSPACE;
    const IndexParams ip = make_index_params(*shape, *spec, seed);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Partial* ws = partials_of(workspace);
    // the dx pass reads x on the points of S only: worth keeping in cache when that is most of the tensor
    const bool x_again = 2u * uint64_t(ip.shared.n_cnt) * uint64_t(ip.shared.h_cnt) * uint64_t(ip.shared.w_cnt) >=
                         uint64_t(d.N) * uint64_t(d.HW);
    if (nhwc(d)) {
        if (g_tuning.path == 2) return BNS_EUNSUPPORTED;
        hipError_t se = hipSuccess;
        if (launch_nhwc_small_backward(d, ip.shared, x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta, st, &se)) {
            t_last_path_backward = 3;
            return dev(se);
        }
        t_last_path_backward = 1;
        // Eq. 6 outside S needs none of the sums: the reduction kernel can write dx there while it has dy in
        // registers, which leaves only the rows of S for after the sums and saves one read of dy from memory.  Only on
        // request: the dx pass finds most of dy in the memory-side cache, and that second read costs less than the
        // slower kernel that the split makes of the reduction (measured up to 128 x 256 x 56 x 56).
        if (g_tuning.nhwc_split_dx == 1) {
            t_last_path_backward = 4;
            return dev(launch_nhwc_backward_split(d, ip.shared, x, dy, gamma, save_mean, save_invstd, ws, dgamma, dbeta, dx, st));
        }
        if (launch_nhwc_reduce(d, x, dy, save_mean, save_invstd, ws, dgamma, dbeta, x_again, st) != hipSuccess)
            return BNS_EDEVICE;
        return dev(launch_nhwc_dx(d, ip.shared, x, dy, gamma, save_mean, save_invstd, dgamma, dbeta, dx, st));
    }
    if (g_tuning.path != 1) {
        FusedIo io;
        io.x = x;
        io.dy = dy;
        io.out = dx;
        io.gamma = gamma;
        io.save_mean = const_cast<float*>(save_mean);
        io.save_invstd = const_cast<float*>(save_invstd);
        io.dgamma = dgamma;
        io.dbeta = dbeta;
        const hipError_t fe = launch_fused(d, ip, true, io, 0.f, 0.f, workspace, slots_of(workspace, d),
                                           kSlotBytes, 0, d.C, st, nullptr, order_streams);
        if (fe == hipSuccess) {
            t_last_path_backward = 2;
            return BNS_OK;
        }
        if (fe != hipErrorNotSupported) return BNS_EDEVICE;
        if (g_tuning.path == 2) return BNS_EUNSUPPORTED;
    }
    t_last_path_backward = 1;
    const int G = channel_group(d);
    for (int c0 = 0; c0 < d.C; c0 += G) {
        const int cg = (d.C - c0 < G) ? d.C - c0 : G;
        s = reduce_range(d, x, dy, save_mean, save_invstd, dgamma, dbeta, ws, c0, cg, x_again, st);
        if (s != BNS_OK) return s;
        s = dev(launch_dx(d, ip, x, dy, gamma, save_mean, save_invstd, dgamma, dbeta, dx, c0, cg, st));
        if (s != BNS_OK) return s;
    }
    return BNS_OK;
}

// Scratch memory of bns_backward_builtin_workspace: one copy per device, held from the moment the library's code
// is loaded on that device until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels and copies take the address that call returns.
constexpr int kMaxDevices = 16;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Address of this device's copy of `scratch` (looked up once per device, with that device current).
bns_status builtin_workspace(void** out) {
    int devid = -1;
    if (hipGetDevice(&devid) != hipSuccess) return BNS_EDEVICE;
    if (devid < 0 || devid >= kMaxDevices) return BNS_EUNSUPPORTED;
    void* p = g_scratch_ptr[devid].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BNS_EDEVICE;
        g_scratch_ptr[devid].store(p, std::memory_order_release);     // every thread finds the same address
    }
    *out = p;
    return BNS_OK;
}
}  // namespace

bns_status bns_backward(const bns_shape* shape, const bns_spec* spec, uint64_t seed, const void* x, const void* dy,
                        const float* gamma, const float* save_mean, const float* save_invstd, void* dx,
                        float* dgamma, float* dbeta, void* workspace, size_t workspace_bytes, void* stream) {
    return backward_impl(shape, spec, seed, x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta, workspace,
                         workspace_bytes, stream, true);
}

bns_status bns_backward_builtin_workspace(const bns_shape* shape, const bns_spec* spec, uint64_t seed, const void* x,
                                          const void* dy, const float* gamma, const float* save_mean,
                                          const float* save_invstd, void* dx, float* dgamma, float* dbeta,
                                          void* stream) {
    Dims d;
    const bns_status s = backward_check(shape, spec, x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta, &d);
    if (s != BNS_OK) return s;
    if (workspace_need(d) > kBuiltinWorkspaceBytes) return BNS_EWORKSPACE;     // too many channels for the built-in scratch
    void* ws = nullptr;
    const bns_status ws_status = builtin_workspace(&ws);
    if (ws_status != BNS_OK) return ws_status;
    // (no event between streams here: creating one allocates, and these calls are ordered by the caller anyway)
    return backward_impl(shape, spec, seed, x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta, ws,
                         kBuiltinWorkspaceBytes, stream, false);
}

// ---- "VDN + sampling", Eq. 4 ---------------------------------------------------------------
namespace {
bns_status check_mixed(const bns_shape* shape, const bns_spec* spec, int32_t n_v, float mix_beta, Dims* d) {
    bns_status s = check_shape(shape, d);
    if (s != BNS_OK) return s;
    if (!spec || n_v < 1 || n_v >= shape->N) return BNS_EINVAL;
    if (!(mix_beta >= 0.f && mix_beta <= 1.f)) return BNS_EINVAL;
    if (spec->mode == BNS_VDN) return BNS_EINVAL;            // the real part needs a sampling strategy
    bns_shape real = *shape;
    real.N = shape->N - n_v;
    return check_spec(&real, spec);
}
}  // namespace

bns_status bns_sample_index_mixed(const bns_shape* shape, const bns_spec* spec, uint64_t seed, int32_t n_v,
                                  bns_box* boxes) {
    Dims d;
    bns_status s = check_mixed(shape, spec, n_v, 0.5f, &d);
    if (s != BNS_OK) return s;
    if (!boxes) return BNS_EINVAL;
    const IndexParams ip = make_index_params_mixed(*shape, *spec, seed, n_v);
    for (int c = 0; c < d.C; ++c) boxes[c] = box_of_channel(ip, c);
    return BNS_OK;
}

bns_status bns_forward_mixed(const bns_shape* shape, const bns_spec* spec, uint64_t seed, int32_t n_v, float mix_beta,
                             const void* x, const float* gamma, const float* beta, float eps, float momentum,
                             void* y, float* save_mean, float* save_invstd, float* save_mean_parts,
                             float* running_mean, float* running_var, void* workspace, size_t workspace_bytes,
                             void* stream) {
    Dims d;
    bns_status s = check_mixed(shape, spec, n_v, mix_beta, &d);
    if (s != BNS_OK) return s;
    if (!x || !gamma || !beta || !y || !save_mean || !save_invstd || !save_mean_parts || !workspace) return BNS_EINVAL;
    if (!aligned16(x) || !aligned16(y) || !aligned16(workspace)) return BNS_EINVAL;
    if (overlap(x, tensor_bytes(d), y, tensor_bytes(d))) return BNS_EINVAL;
    if (!(eps >= 0.f) || !(momentum >= 0.f && momentum <= 1.f)) return BNS_EINVAL;
    if (workspace_bytes < workspace_need(d)) return BNS_EWORKSPACE;
    if ((s = check_layout(d, spec)) != BNS_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const IndexParams ip_s = make_index_params_mixed(*shape, *spec, seed, n_v);
    if (nhwc(d)) {
        if (g_tuning.path == 2) return BNS_EUNSUPPORTED;
        t_last_path_forward = 1;
        if (launch_nhwc_stats_mixed(d, ip_s.shared, n_v, x, partials_of(workspace), mix_beta, eps, momentum,
                                    save_mean, save_invstd, save_mean_parts, running_mean, running_var, st) != hipSuccess)
            return BNS_EDEVICE;
        return dev(launch_nhwc_normalize(d, x, gamma, beta, save_mean, save_invstd, y, st));
    }
    if (g_tuning.path != 1) {
        FusedIo io;
        io.x = x;
        io.out = y;
        io.gamma = gamma;
        io.beta = beta;
        io.save_mean = save_mean;
        io.save_invstd = save_invstd;
        io.running_mean = running_mean;
        io.running_var = running_var;
        FusedMix mix;
        mix.n_v = n_v;
        mix.mix_beta = mix_beta;
        mix.mean_parts = save_mean_parts;
        const hipError_t fe = launch_fused(d, ip_s, false, io, eps, momentum,
                                           workspace, slots_of(workspace, d), kSlotBytes, 0, d.C, st,
                                           &mix);
        if (fe == hipSuccess) {
            t_last_path_forward = 2;
            return BNS_OK;
        }
        if (fe != hipErrorNotSupported) return BNS_EDEVICE;
        if (g_tuning.path == 2) return BNS_EUNSUPPORTED;
    }
    t_last_path_forward = 1;
    const IndexParams ip_v = make_index_params_virtual(*shape, n_v);
    Partial* ws_s = partials_of(workspace);
    Partial* ws_v = reinterpret_cast<Partial*>(reinterpret_cast<char*>(partials_of(workspace)) + partial_bytes(d));
    const int splits_s = stats_splits(d, ip_s, d.C);
    const int splits_v = stats_splits(d, ip_v, d.C);
    if (launch_stats_partial(d, ip_s, x, ws_s, splits_s, 0, d.C, st) != hipSuccess) return BNS_EDEVICE;
    if (launch_stats_partial(d, ip_v, x, ws_v, splits_v, 0, d.C, st) != hipSuccess) return BNS_EDEVICE;
    if (launch_stats_finalize_mixed(d, ip_s, ip_v, x, ws_s, splits_s, ws_v, splits_v, mix_beta, eps, momentum, save_mean,
                                    save_invstd, save_mean_parts, running_mean, running_var, st) != hipSuccess)
        return BNS_EDEVICE;
    return dev(launch_normalize(d, x, gamma, beta, save_mean, save_invstd, y, 0, d.C, st));
}

bns_status bns_backward_mixed(const bns_shape* shape, const bns_spec* spec, uint64_t seed, int32_t n_v, float mix_beta,
                              const void* x, const void* dy, const float* gamma, const float* save_mean,
                              const float* save_invstd, const float* save_mean_parts, void* dx, float* dgamma,
                              float* dbeta, void* workspace, size_t workspace_bytes, void* stream) {
    Dims d;
    bns_status s = check_mixed(shape, spec, n_v, mix_beta, &d);
    if (s != BNS_OK) return s;
    if (!x || !dy || !gamma || !save_mean || !save_invstd || !save_mean_parts || !dx || !dgamma || !dbeta || !workspace)
        return BNS_EINVAL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) || !aligned16(workspace)) return BNS_EINVAL;
    const size_t tb = tensor_bytes(d);
    if (overlap(dx, tb, x, tb) || overlap(dx, tb, dy, tb)) return BNS_EINVAL;
    if (workspace_bytes < workspace_need(d)) return BNS_EWORKSPACE;
    if ((s = check_layout(d, spec)) != BNS_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const IndexParams ip_s = make_index_params_mixed(*shape, *spec, seed, n_v);
    if (nhwc(d)) {
        if (g_tuning.path == 2) return BNS_EUNSUPPORTED;
        t_last_path_backward = 1;
        if (launch_nhwc_reduce(d, x, dy, save_mean, save_invstd, partials_of(workspace), dgamma, dbeta, false, st) !=
            hipSuccess)
            return BNS_EDEVICE;
        return dev(launch_nhwc_dx_mixed(d, ip_s.shared, n_v, mix_beta, x, dy, gamma, save_invstd, dgamma, dbeta,
                                        save_mean_parts, dx, st));
    }
    if (g_tuning.path != 1) {
        FusedIo io;
        io.x = x;
        io.dy = dy;
        io.out = dx;
        io.gamma = gamma;
        io.save_mean = const_cast<float*>(save_mean);
        io.save_invstd = const_cast<float*>(save_invstd);
        io.dgamma = dgamma;
        io.dbeta = dbeta;
        FusedMix mix;
        mix.n_v = n_v;
        mix.mix_beta = mix_beta;
        mix.mean_parts = const_cast<float*>(save_mean_parts);
        const hipError_t fe = launch_fused(d, ip_s, true, io, 0.f, 0.f, workspace, slots_of(workspace, d),
                                           kSlotBytes, 0, d.C, st, &mix);
        if (fe == hipSuccess) {
            t_last_path_backward = 2;
            return BNS_OK;
        }
        if (fe != hipErrorNotSupported) return BNS_EDEVICE;
        if (g_tuning.path == 2) return BNS_EUNSUPPORTED;
    }
    t_last_path_backward = 1;
    s = reduce_range(d, x, dy, save_mean, save_invstd, dgamma, dbeta, partials_of(workspace), 0, d.C, false, st);
    if (s != BNS_OK) return s;
    const bns_box& b = ip_s.shared;
    DxSets sets;
    sets.n_v = n_v;
    sets.w_s = float((1.0 - double(mix_beta)) / (double(b.n_cnt) * double(b.h_cnt) * double(b.w_cnt)));
    sets.w_v = float(double(mix_beta) / (double(n_v) * double(d.HW)));
    sets.centre_v = save_mean_parts;
    sets.centre_s = save_mean_parts + d.C;
    return dev(launch_dx(d, ip_s, x, dy, gamma, save_mean, save_invstd, dgamma, dbeta, dx, 0, d.C, st, &sets));
}

bns_status bns_expired_waits(void* workspace, size_t workspace_bytes, void* stream, int32_t* expired) {
    if (!expired) return BNS_EINVAL;
    void* ws = workspace;
    if (!ws) {                                              // the built-in scratch of bns_backward_builtin_workspace
        const bns_status s = builtin_workspace(&ws);
        if (s != BNS_OK) return s;
    } else if (!aligned16(ws)) {
        return BNS_EINVAL;
    } else if (workspace_bytes < kHeaderBytes) {
        return BNS_EWORKSPACE;
    }
    return dev(read_expired_waits(ws, static_cast<hipStream_t>(stream), expired));
}

float bns_moving_average_weight(uint64_t iteration, float alpha) { return iteration <= 1 ? 1.0f : alpha; }   // Eq. 8

bns_status bns_copy_reference(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || (bytes & 15u) || !aligned16(dst) || !aligned16(src)) return BNS_EINVAL;
    if ((bytes / 16 + 1023) / 1024 >= (size_t(1) << 31)) return BNS_EUNSUPPORTED;
    if (overlap(dst, bytes, src, bytes)) return BNS_EINVAL;
    return dev(launch_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
}

bns_status bns_set_option(const char* name, int32_t value) {
    if (!name || value < 0) return BNS_EINVAL;
    if (!strcmp(name, "splits_stats") || !strcmp(name, "splits_reduce")) {
        if (value > kMaxSplits) return BNS_EINVAL;
        (name[7] == 's' ? g_splits_stats : g_splits_reduce).store(value);
        return BNS_OK;
    }
    if (!strcmp(name, "channel_group")) {
        g_channel_group.store(value);
        return BNS_OK;
    }
    for (const TuningEntry& t : kTuningTable)
        if (!strcmp(name, t.name)) {
            if (value > t.hi || (t.pow2 && value == 3)) return BNS_EINVAL;
            g_tuning.*(t.field) = value - t.bias;
            return BNS_OK;
        }
    return BNS_EINVAL;
}

int32_t bns_get_option(const char* name) {
    if (!name) return -1;
    if (!strcmp(name, "splits_stats")) return g_splits_stats.load();
    if (!strcmp(name, "splits_reduce")) return g_splits_reduce.load();
    if (!strcmp(name, "channel_group")) return g_channel_group.load();
    if (!strcmp(name, "last_path_forward")) return t_last_path_forward;
    if (!strcmp(name, "last_path_backward")) return t_last_path_backward;
    if (!strcmp(name, "last_fused_backward")) return t_last_fused_backward;
    if (!strcmp(name, "last_fused_forward")) return t_last_fused_forward;
    if (!strcmp(name, "launch_count")) return int32_t(g_launch_count.load() & 0x7fffffffu);
    for (const TuningEntry& t : kTuningTable)
        if (!strcmp(name, t.name)) {
            const int v = g_tuning.*(t.field) + t.bias;         // as it was set; 0 = automatic
            return v < 0 ? 0 : v;
        }
    return -1;
}

}  // extern "C"
