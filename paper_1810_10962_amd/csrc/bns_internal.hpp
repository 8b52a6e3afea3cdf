// Host-side launch interface between the C ABI (bns_api.hip) and the kernels
// (bns_kernels.hip).  Every launcher works on the channel range [c0, c0 + cg).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "bns_index.hpp"
#include "bns_validate.hpp"

// Kernel launch whose status the following hipGetLastError() reports: the thread's last-error state may
// still hold a failure of some earlier, unrelated runtime call (the caller's, the framework's), which must
// not be taken for this launch's, so it is cleared first.
#define BNS_LAUNCH(...)                                              \
    do {                                                             \
        (void)hipGetLastError();                                     \
        ::bns::g_launch_count.fetch_add(1, std::memory_order_relaxed); \
        hipLaunchKernelGGL(__VA_ARGS__);                             \
    } while (0)

namespace bns {

// Kernels launched by the library since it was loaded ("launch_count" option: benchmarks report launches per call).
extern std::atomic<uint32_t> g_launch_count;
// Which single-launch backward kernel the calling thread's last fused backward call took: 1 plain, 2 x kept in registers, 3 pipelined.
extern thread_local int32_t t_last_fused_backward;
// Which flavour the calling thread's last fused forward call took: 1 plain or patch elements read on their own,
// 2 patch statistics from the registers.
extern thread_local int32_t t_last_fused_forward;

constexpr int kMaxSplits = 64;  // upper bound on blocks that share one channel's reduction


// Launch-shape choices; 0 = the default for the storage type (see tuned()).  The benchmark
// can override them through bns_set_option.  Defaults come from sweeps on MI355X at
// 64x256x56x56: one 128-bit access per thread and non-temporal loads and stores stream
// fastest (keeping streamed data out of the caches avoids write-backs of lines nobody will
// hit); the exception is data that the very next pass reads again, see keep_for_next_pass.
// Every field is an atomic: bns_set_option may run while another thread launches work (that call then
// sees the old or the new value of each field it reads, never a torn one).
using TuneInt = std::atomic<int>;
struct Tuning {
    TuneInt norm_unroll{0}, norm_nt{-1};    // accesses per thread; bit 0: non-temporal loads, bit 1: stores
    TuneInt dx_unroll{0}, dx_nt{-1};
    TuneInt reduce_unroll{0}, reduce_nt{-1};    // reduce_nt: bit 0 non-temporal loads of x, bit 1 of dy
    TuneInt cache_reuse{0};                 // a first pass loads what the next pass reads again so that it stays in the
                                            // memory-side cache: 1 always, 2 never, 0 when it fits (kKeepBytes)
    TuneInt path{0};                        // 0: fused kernels when a channel fits on chip, else streaming;
                                            // 1: streaming kernels only; 2: fused only (error if it cannot)
    TuneInt fused_variant{0};               // 1..7 forces a (block size, registers) variant of the fused kernels
    TuneInt fused_keep_x{0};                // backward keeps x in registers next to dy: 1 always, 2 never, 0 when it pays
    TuneInt fused_pipe{0};                  // backward: 1..n forces variant n of the pipelined kernel, 16: never
    TuneInt fused_team{0};                  // blocks per team of the pipelined kernel, if the channel fits (0: planner)
    TuneInt fused_patch_mask{0};            // forward, patch: statistics from the registers 1 = whenever built, 2 = never, 0 = when a block holds its channel alone
    TuneInt fused_coop{0};                  // 1: launch the fused kernels with hipLaunchCooperativeKernel
    TuneInt split_statistics{0};            // 1: forward statistics always as partial sums + finalize
    TuneInt nhwc_blocks{0};                 // blocks an N x H x W x C reduction aims for (default kNhwcBlocks)
    TuneInt nhwc_small{0};                  // 2: never take the one-launch kernels for small N x H x W x C tensors
    TuneInt nhwc_ew_rows{0};                // rows per row lane in its element-wise kernels (default kNhwcEwRows)
    TuneInt nhwc_split_dx{0};               // backward writes dx outside S from the reduction kernel: 1 always, 2 never, 0 when S is at most half
    // For the library's own tests of the give-up path only; a caller has no use for them.
    TuneInt test_spin_limit{0};             // polls a team member waits for a team-mate before giving up (default 2^21)
    TuneInt test_mute_exchange{0};          // 1: no member publishes its sums, so every wait runs out
};
extern Tuning g_tuning;
inline int tuned(int v, int dflt) { return v > 0 ? v : dflt; }
inline int tuned_nt(int v, int dflt) { return v >= 0 ? v : dflt; }

// Two passes over one tensor (statistics then Eq. 1; the sums of Eq. 5 then Eq. 6): the second pass finds in the
// 256 MB memory-side cache what the first one loaded without the non-temporal hint, which for a copy-like pass is
// worth about a quarter of its time (reads served there leave the memory to the writes).  Plain loads stream
// some 10 % slower than non-temporal ones, so a first pass uses them only for what fits, with room to spare for
// the other traffic of the two passes.
constexpr size_t kKeepBytes = size_t(224) << 20;
inline bool keep_for_next_pass(size_t bytes) {
    const int o = g_tuning.cache_reuse;
    return o == 1 || (o == 0 && bytes <= kKeepBytes);
}

// One (sum, sum) pair per channel and split.
struct Partial {
    float a, b;
};

// Forward statistics (Eq. 3): partial sums of (x - pivot) and (x - pivot)^2 over S.
hipError_t launch_stats_partial(const Dims& d, const IndexParams& ip, const void* x, Partial* partial,
                                int splits, int c0, int cg, hipStream_t st);
// Statistics and Eq. 8 in one launch with one 1024-thread block per channel, for channels with few
// sampled points; returns false (nothing launched) when that does not apply.
bool launch_stats_one_block(const Dims& d, const IndexParams& ip, const void* x, int c0, int cg, float eps,
                            float momentum, float* save_mean, float* save_invstd, float* running_mean,
                            float* running_var, hipStream_t st, hipError_t* err);
// Fixed-order combine, mean / inv-std, running averages (Eq. 8).
hipError_t launch_stats_finalize(const Dims& d, const IndexParams& ip, const void* x, const Partial* partial,
                                 int splits, int c0, int cg, float eps, float momentum,
                                 float* save_mean, float* save_invstd, float* running_mean,
                                 float* running_var, hipStream_t st);
// Eq. 1 over every element.  var_eps >= 0: `invstd` holds variances and 1/sqrt(var + var_eps) is used.
hipError_t launch_normalize(const Dims& d, const void* x, const float* gamma, const float* beta,
                            const float* mean, const float* invstd, void* y, int c0, int cg, hipStream_t st,
                            float var_eps = -1.f);
// Backward sums of Eq. 5 over all m points: partial sums of dy and dy * (x - mean).
// x_again: the dx pass reads every element of x again (S is everything), not only those of a small S
hipError_t launch_reduce_partial(const Dims& d, const void* x, const void* dy, const float* mean,
                                 Partial* partial, int splits, int c0, int cg, bool x_again, hipStream_t st);
hipError_t launch_reduce_finalize(const Dims& d, const Partial* partial, int splits, int c0, int cg,
                                  const float* invstd, float* dgamma, float* dbeta, hipStream_t st);
// Which 1/s terms an element receives in the dx pass.  Plain sampled BN: one set, weight 1/s,
// centred on the saved mean.  "VDN + sampling" (Eq. 4): samples below n_v form the virtual set
// (weight beta_mix / s_v, centre E_v), the index describes the sampled real set (weight
// (1 - beta_mix) / s_s, centre E_s).
struct DxSets {
    int32_t n_v = 0;
    float w_s = 0.f, w_v = 0.f;
    const float* centre_s = nullptr;
    const float* centre_v = nullptr;
};
// Eq. 6 over every element.
hipError_t launch_dx(const Dims& d, const IndexParams& ip, const void* x, const void* dy, const float* gamma,
                     const float* mean, const float* invstd, const float* dgamma, const float* dbeta,
                     void* dx, int c0, int cg, hipStream_t st, const DxSets* sets = nullptr);
// Eq. 4: combine the partial sums of the virtual set and of the sampled real set.
hipError_t launch_stats_finalize_mixed(const Dims& d, const IndexParams& ip_s, const IndexParams& ip_v, const void* x,
                                       const Partial* partial_s, int splits_s, const Partial* partial_v,
                                       int splits_v, float mix_beta, float eps, float momentum, float* save_mean,
                                       float* save_invstd, float* mean_parts, float* running_mean,
                                       float* running_var, hipStream_t st);

// Fused single-launch passes (bns_fused.hip).  Pointers a pass does not use are null.
struct FusedIo {
    const void* x = nullptr;
    const void* dy = nullptr;
    void* out = nullptr;
    const float* gamma = nullptr;
    const float* beta = nullptr;
    float* save_mean = nullptr;
    float* save_invstd = nullptr;
    float* running_mean = nullptr;
    float* running_var = nullptr;
    float* dgamma = nullptr;
    float* dbeta = nullptr;
};
constexpr size_t kSlotBytes = 256 * 1024;   // stamped exchange slots of the fused kernels
constexpr size_t kHeaderBytes = 256;        // in front of everything else in a workspace
// hipErrorNotSupported: the channel does not fit on chip (take the streaming kernels instead).
// mix != nullptr: "VDN + sampling" (Eq. 4); `ip` then describes the sampled real set.
struct FusedMix {
    int32_t n_v = 0;
    float mix_beta = 0.f;
    float* mean_parts = nullptr;     // [E_v per channel][E_s per channel]: forward writes, backward reads
};
// header: the first kHeaderBytes of the workspace (launch counter, count of waits that ran out).
// order_streams: chain launches whose blocks wait for each other across streams with an event (see there).
hipError_t launch_fused(const Dims& d, const IndexParams& ip, bool backward, const FusedIo& io, float eps,
                        float momentum, void* header, void* slots, size_t slot_bytes, int c0, int cg, hipStream_t st,
                        const FusedMix* mix = nullptr, bool order_streams = true);
// Reads the count of waits that ran out from a workspace header (0 if the header was never set up) and clears it.
hipError_t read_expired_waits(void* header, hipStream_t st, int32_t* expired);

hipError_t launch_index_boxes(const IndexParams& ip, int C, bns_box* boxes, hipStream_t st);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st);

// Blocks per channel for a reduction over `vectors_per_channel` memory accesses.
int auto_splits(int cg, uint32_t vectors_per_channel);

// N x H x W x C layout (bns_nhwc.hip): streaming kernels over all channels; `b` is the one location
// set shared by the channels.  Partial sums: nhwc_partial_bytes(d) bytes of workspace.
constexpr int kNhwcBlocks = 512;       // blocks a reduction launch aims for (2 per compute unit: measured best)
constexpr int kNhwcFill = 2048;        // fewest blocks an element-wise launch aims for (8 per compute unit)
constexpr int kNhwcBlocksMax = 8192;   // largest value the "nhwc_blocks" override takes
constexpr int kNhwcEwRows = 4;         // rows per row lane and block in the element-wise kernels
constexpr int kNhwcMaxSplits = 2048;   // upper bound on blocks that share one channel's reduction
constexpr int kNhwcSmallRows = 16;     // rows per row lane up to which one block walks all rows of its channels
constexpr int kNhwcMaxLaneRows = 1024; // rows one thread accumulates in fp32 before the sums are combined
size_t nhwc_partial_bytes(const Dims& d);
hipError_t launch_nhwc_stats(const Dims& d, const bns_box& b, const void* x, Partial* partial, float eps, float momentum,
                             float* save_mean, float* save_invstd, float* running_mean, float* running_var,
                             hipStream_t st);
hipError_t launch_nhwc_normalize(const Dims& d, const void* x, const float* gamma, const float* beta, const float* mean,
                                 const float* invstd, void* y, hipStream_t st, float var_eps = -1.f);
// x_again: as for launch_reduce_partial
hipError_t launch_nhwc_reduce(const Dims& d, const void* x, const void* dy, const float* mean, const float* invstd,
                              Partial* partial, float* dgamma, float* dbeta, bool x_again, hipStream_t st);
// Backward with dx split by the two branches of Eq. 6: the reduction kernel also writes dx outside S, a second
// element-wise kernel takes the rows of S after the sums ((3 + 2r) e bytes per element instead of (4 + r) e).
hipError_t launch_nhwc_backward_split(const Dims& d, const bns_box& b, const void* x, const void* dy, const float* gamma,
                                      const float* mean, const float* invstd, Partial* partial, float* dgamma,
                                      float* dbeta, void* dx, hipStream_t st);
hipError_t launch_nhwc_dx(const Dims& d, const bns_box& b, const void* x, const void* dy, const float* gamma,
                          const float* mean, const float* invstd, const float* dgamma, const float* dbeta, void* dx,
                          hipStream_t st);
// Eq. 4 in this layout: statistics of the sampled real set and of the first n_v samples, blended; dx with
// per-set weights.  `partial` then holds two regions of nhwc_partial_bytes(d).
hipError_t launch_nhwc_stats_mixed(const Dims& d, const bns_box& b, int n_v, const void* x, Partial* partial,
                                   float mix_beta, float eps, float momentum, float* save_mean, float* save_invstd,
                                   float* mean_parts, float* running_mean, float* running_var, hipStream_t st);
hipError_t launch_nhwc_dx_mixed(const Dims& d, const bns_box& b, int n_v, float mix_beta, const void* x, const void* dy,
                                const float* gamma, const float* invstd, const float* dgamma, const float* dbeta,
                                const float* mean_parts, void* dx, hipStream_t st);
// Whole forward / backward in one launch for small tensors; false (nothing launched) when the tensor is not small.
bool launch_nhwc_small_forward(const Dims& d, const bns_box& b, const void* x, const float* gamma, const float* beta,
                               float eps, float momentum, void* y, float* save_mean, float* save_invstd,
                               float* running_mean, float* running_var, hipStream_t st, hipError_t* err);
bool launch_nhwc_small_backward(const Dims& d, const bns_box& b, const void* x, const void* dy, const float* gamma,
                                const float* mean, const float* invstd, void* dx, float* dgamma, float* dbeta,
                                hipStream_t st, hipError_t* err);

}  // namespace bns
