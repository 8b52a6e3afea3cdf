/* libbns -- sampled batch normalisation for AMD MI355X (gfx950).
 *
 * Training-mode batch normalisation, forward and backward, in which the
 * per-channel mean and variance are estimated from a sampled subset S of the
 * activations ("Batch Normalization Sampling", Chen, Deng, Li et al.,
 * arXiv 1810.10962).  Citations below are to that paper.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Layout     x, y, dy, dx are dense tensors, element type given by
 *            bns_shape.dtype, in the layout bns_shape.layout names: N x C x H x W
 *            (channel planes of H*W contiguous elements; the default) or
 *            N x H x W x C (channels contiguous, the layout the paper's notation
 *            uses, Appendix A).  Either way the reduction axes are N, H, W, the
 *            paper's E_{0,1,2} / Var_{0,1,2}, and the same (shape, spec, seed) give
 *            the same index and, up to rounding order, the same results.
 *            Per-channel vectors (gamma, beta, statistics, dgamma, dbeta) are
 *            float[C].
 * Memory     Unless an argument is marked HOST it is a DEVICE pointer owned by
 *            the caller, at least 16-byte aligned.  The library allocates and
 *            frees nothing and keeps no state between calls except the tuning
 *            overrides of bns_set_option.  `workspace` is caller-provided
 *            device scratch of at least bns_workspace_bytes() bytes; its
 *            contents need not be initialised.  Its first 256 bytes hold a launch
 *            counter that the single-launch kernels keep from call to call: a
 *            workspace may be overwritten between calls (the counter is set up
 *            again), but not while a call that uses it is running.
 * Streams    `stream` is a hipStream_t passed as void* (NULL = the default
 *            stream).  Work is enqueued on it and the call returns without
 *            synchronising.  Calls that share a workspace must be ordered on
 *            one stream.
 * Concurrency The single-launch ("fused") kernels size their grid to what the
 *            device holds at once and let the blocks that share a channel wait
 *            for each other.  Calls from several host threads and streams of one
 *            process are safe: the library chains such kernels with an event, so
 *            that two of them never share the device.  If work the library does not
 *            know of occupies the device at the same time (another process, a HIP
 *            graph that holds captured libbns calls and is replayed beside other
 *            libbns calls), a wait can last until that work ends; it is bounded
 *            (2^21 polls, then 2^15 for the rest of the launch), after which the
 *            results of that channel are NaN -- never a wrong finite value -- the
 *            moving averages keep their old values, the kernel ends normally, and
 *            bns_expired_waits() reports it, so nobody has to scan tensors.
 * Aliasing   Outputs must not overlap inputs or each other (x is needed again
 *            by the backward pass; dx is written while dy is read).  The host
 *            checks the tensors (y against x; dx against x and dy) and returns
 *            BNS_EINVAL when they overlap.  The per-channel vectors and the
 *            workspace are not checked against anything: keeping them apart
 *            from each other and from the tensors is the caller's duty.
 * Errors     Every call returns a bns_status.  Arguments are validated on the
 *            host before anything is enqueued: BNS_EINVAL for NULL pointers,
 *            non-positive extents, n_s outside [1, N] (Alg. 1), patch sizes
 *            outside [1, H] x [1, W] (Alg. 2), VDN with n_s >= N, unknown
 *            enums, misaligned pointers, an output tensor that overlaps an
 *            input tensor (see Aliasing);
 *            BNS_EUNSUPPORTED for extents beyond the limits listed at
 *            bns_shape; BNS_EWORKSPACE when the workspace is too small;
 *            BNS_EDEVICE when the HIP runtime reports a launch failure.
 *            Nothing is thrown across the boundary.
 * Determinism No floating-point atomics: per-channel sums are combined in a
 *            fixed order, so results are bit-identical from run to run.
 */
#ifndef BNS_H
#define BNS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BNS_OK = 0,
    BNS_EINVAL = 1,
    BNS_EUNSUPPORTED = 2,
    BNS_EWORKSPACE = 3,
    BNS_EDEVICE = 4
} bns_status;

/* Which activations feed the statistics. */
typedef enum {
    BNS_FULL = 0, /* all m = N*H*W points of a feature map (Eq. 2): plain BN                   */
    BNS_NS = 1,   /* Naive Sampling: samples 0 .. n_s-1 (Alg. 1 with begin = 0)                */
    BNS_BS = 2,   /* Batch Sampling: samples begin .. begin+n_s-1, begin = randint(0, N-n_s),
                     one draw per (layer, epoch), shared by all channels (Alg. 1, Sec. 4.1)    */
    BNS_FS = 3,   /* Feature Sampling: one patch_h x patch_w patch at (begin_h, begin_w) of
                     every sample (Alg. 2); one location per layer, or one per channel         */
    BNS_VDN = 4   /* Virtual Dataset Normalisation: the n_s virtual samples that the caller
                     concatenated in front of the batch, samples 0 .. n_s-1 (Alg. 3)           */
} bns_mode;

typedef enum { BNS_F32 = 0, BNS_BF16 = 1 } bns_dtype; /* storage of x, y, dy, dx; arithmetic is fp32 */

typedef enum { BNS_NCHW = 0, BNS_NHWC = 1 } bns_layout; /* memory order of x, y, dy, dx */

/* Tensor extents.  For VDN, N counts virtual + real samples (virtual first).
 * Limits: N <= 65535, C <= 2^24, H*W < 2^31, N*H*W < 2^31, C*H*W < 2^31.
 * BNS_NHWC: every channel shares one location set there, so Feature Sampling with
 * fs_per_channel = 1 returns BNS_EUNSUPPORTED; the other modes, the bns_*_mixed calls, both storage
 * types and every stage call are available. */
typedef struct {
    int32_t N, C, H, W;
    int32_t dtype;  /* bns_dtype */
    int32_t layout; /* bns_layout */
} bns_shape;

/* Sampling specification.  (seed, layer_id, epoch) select the random index: the paper
 * refreshes indices once per epoch and draws them independently per layer (Sec. 4.1). */
typedef struct {
    int32_t mode;             /* bns_mode */
    int32_t n_s;              /* NS/BS: samples kept; VDN: number of virtual samples; else ignored */
    int32_t patch_h, patch_w; /* FS: patch extent; else ignored */
    int32_t fs_per_channel;   /* FS: 0 = one patch location per layer (the paper's rule),
                                 1 = an independent location for each channel */
    uint32_t layer_id;
    uint32_t epoch;
} bns_spec;

/* The location set S of one channel: the box [n0, n0+n_cnt) x [h0, h0+h_cnt) x [w0, w0+w_cnt). */
typedef struct {
    int32_t n0, n_cnt, h0, h_cnt, w0, w_cnt;
} bns_box;

const char* bns_status_string(bns_status s);

/* Sampling index, computed on the host (Alg. 1-3; "randint" includes both ends).
 * boxes: HOST array of shape->C entries, written.  A pure integer function of
 * (shape, spec, seed): 64-bit SplitMix64-style mixing of seed, layer_id, epoch, the
 * coordinate being drawn and (per-channel FS only) the channel; the top 32 bits are
 * scaled to the number of outcomes.  No device is touched. */
bns_status bns_sample_index(const bns_shape* shape, const bns_spec* spec, uint64_t seed,
                            bns_box* boxes /* HOST, C entries */);

/* The same index evaluated by the generator the kernels use, on the device.
 * boxes: DEVICE array of shape->C entries, written on `stream`. */
bns_status bns_sample_index_device(const bns_shape* shape, const bns_spec* spec, uint64_t seed,
                                   bns_box* boxes /* DEVICE, C entries */, void* stream);

/* Bytes of device scratch that bns_forward / bns_backward and their stages need (depends on the
 * extents and the layout only). */
size_t bns_workspace_bytes(const bns_shape* shape, const bns_spec* spec);

/* Forward (Eq. 1 with the statistics of Eq. 3):
 *   save_mean[c]   = E    = mean of x over S_c
 *   save_invstd[c] = 1 / sqrt(Var + eps), Var = biased variance of x over S_c
 *   y = gamma * (x - E) * invstd + beta                       for all N*H*W points
 *   running_mean/var <- (1 - momentum) * running + momentum * (E | Var)     (Eq. 8; pass
 *   momentum = 1 for its first-iteration branch); either may be NULL = not kept.
 * in: x, gamma, beta.  out: y, save_mean, save_invstd.  in-out: running_*. */
bns_status bns_forward(const bns_shape* shape, const bns_spec* spec, uint64_t seed,
                       const void* x, const float* gamma, const float* beta,
                       float eps, float momentum,
                       void* y, float* save_mean, float* save_invstd,
                       float* running_mean, float* running_var,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Backward (Eq. 5 with the modification of Eq. 6).  With g = dl/dy, r = save_invstd,
 * x^ = (x - save_mean) * r and s = |S_c|:
 *   dbeta[c]  = sum over all m points of g
 *   dgamma[c] = sum over all m points of g * x^
 *   dx_i = gamma r g_i                                            for x_i outside S
 *   dx_i = gamma r (g_i - (dbeta + x^_i dgamma) / s)              for x_i in S
 * (Eq. 6 after substituting dl/dE and dl/dVar of Eq. 5).  The index is re-derived from
 * (spec, seed), which must equal the forward call's.
 * in: x, dy, gamma, save_mean, save_invstd.  out: dx, dgamma, dbeta. */
bns_status bns_backward(const bns_shape* shape, const bns_spec* spec, uint64_t seed,
                        const void* x, const void* dy, const float* gamma,
                        const float* save_mean, const float* save_invstd,
                        void* dx, float* dgamma, float* dbeta,
                        void* workspace, size_t workspace_bytes, void* stream);

/* bns_backward for callers that cannot hand over a workspace they allocated: code recorded into a HIP graph
 * whose buffers are fixed before the scratch size is known, tight serving or training loops, harnesses that
 * forbid hipMalloc.  Same arguments, results (bit for bit) and errors as bns_backward, without `workspace`:
 * the partial sums and exchange slots live in an array of 4 MiB + 256 bytes built into the library's device code, one copy
 * per GPU, held from the first use of the library on that GPU until the process ends.  The call allocates
 * and frees nothing.  BNS_EWORKSPACE if bns_workspace_bytes(shape, spec) exceeds that size (N x C x H x W: more than
 * 3840 channels).  All such calls on one GPU share the one array, which keeps what the last call left in it
 * (nothing in it has to start at zero): they must be ordered on one stream, like calls that share a
 * workspace; calls that overlap on a GPU race.  The first call on each GPU looks the array's address up and
 * should be made outside stream capture. */
bns_status bns_backward_builtin_workspace(const bns_shape* shape, const bns_spec* spec, uint64_t seed,
                                          const void* x, const void* dy, const float* gamma,
                                          const float* save_mean, const float* save_invstd,
                                          void* dx, float* dgamma, float* dbeta, void* stream);

/* How many waits between blocks of the single-launch kernels ran out (see Concurrency) in the calls that used
 * `workspace` since the last such query; 0 = every result is what the equations say.  Calls whose waits ran
 * out have written NaN to the outputs of the channels concerned.  Synchronises `stream` (the stream those calls
 * were issued to), reads the count from the workspace and clears it; not to be called while `stream` is being
 * captured.  workspace = NULL asks about the built-in scratch of bns_backward_builtin_workspace.
 * expired: HOST, written. */
bns_status bns_expired_waits(void* workspace, size_t workspace_bytes, void* stream, int32_t* expired /* HOST */);

/* The stages that the two calls above are made of, for callers that want to place
 * other work between them (and for per-kernel timing).  Same conventions.
 *
 * bns_forward_stats     Eq. 3 + Eq. 8: statistics of x over S and running averages.
 * bns_forward_normalize Eq. 1: y from x and the saved statistics, all points.
 * bns_backward_reduce   the two length-m sums of Eq. 5: dbeta and dgamma.
 * bns_backward_dx       Eq. 6: dx from dy, (x on S), the statistics and dgamma, dbeta. */
bns_status bns_forward_stats(const bns_shape* shape, const bns_spec* spec, uint64_t seed,
                             const void* x, float eps, float momentum,
                             float* save_mean, float* save_invstd,
                             float* running_mean, float* running_var,
                             void* workspace, size_t workspace_bytes, void* stream);
bns_status bns_forward_normalize(const bns_shape* shape, const void* x,
                                 const float* gamma, const float* beta,
                                 const float* save_mean, const float* save_invstd,
                                 void* y, void* stream);
bns_status bns_backward_reduce(const bns_shape* shape, const void* x, const void* dy,
                               const float* save_mean, const float* save_invstd,
                               float* dgamma, float* dbeta,
                               void* workspace, size_t workspace_bytes, void* stream);
bns_status bns_backward_dx(const bns_shape* shape, const bns_spec* spec, uint64_t seed,
                           const void* x, const void* dy, const float* gamma,
                           const float* save_mean, const float* save_invstd,
                           const float* dgamma, const float* dbeta,
                           void* dx, void* stream);

/* "VDN + sampling" (Sec. 4.2 step 3, Eq. 4).  The tensor holds n_v virtual samples in front of
 * N - n_v real ones (Alg. 3).  `spec` (mode FULL, NS, BS or FS) is the sampling strategy applied to
 * the REAL samples, exactly as Alg. 1 / Alg. 2 on a batch of N - n_v samples shifted by n_v.  With
 * x_v the virtual set and x_s the sampled real set, each statistic by Eq. 3 on its own set,
 *   E   = mix_beta * E[x_v]   + (1 - mix_beta) * E[x_s]
 *   Var = mix_beta * Var[x_v] + (1 - mix_beta) * Var[x_s]           (the paper uses mix_beta = 0.5)
 * save_mean / save_invstd hold the blended E and 1/sqrt(Var + eps); save_mean_parts (float[2*C])
 * holds E[x_v] for every channel, then E[x_s] for every channel: the backward pass centres the
 * variance terms on them.  Everything else as bns_forward.
 * Errors as bns_forward, plus BNS_EINVAL for n_v outside [1, N-1], mix_beta outside [0, 1],
 * mode VDN, or a spec that is invalid for N - n_v samples.  Like bns_forward / bns_backward the two calls
 * take the single-launch kernels when a channel fits on chip and the streaming kernels otherwise
 * ("path" option, "last_path_forward" / "last_path_backward"). */
bns_status bns_sample_index_mixed(const bns_shape* shape, const bns_spec* spec, uint64_t seed, int32_t n_v,
                                  bns_box* boxes /* HOST, C entries: the sampled REAL set */);
bns_status bns_forward_mixed(const bns_shape* shape, const bns_spec* spec, uint64_t seed,
                             int32_t n_v, float mix_beta,
                             const void* x, const float* gamma, const float* beta,
                             float eps, float momentum,
                             void* y, float* save_mean, float* save_invstd, float* save_mean_parts,
                             float* running_mean, float* running_var,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Backward of bns_forward_mixed.  The paper prints none for Eq. 4; by the chain rule, in the form
 * of Eq. 5 / Eq. 6, with g = dl/dy, r = save_invstd, x^ = (x - E) r and dbeta, dgamma the sums over
 * all points as in bns_backward:
 *   dx_i = gamma r g_i - gamma r w (dbeta + r dgamma (x_i - E_set))
 * with (w, E_set) = (mix_beta / s_v, E[x_v]) on the virtual set, ((1 - mix_beta) / s_s, E[x_s]) on
 * the sampled real set, and w = 0 elsewhere. */
bns_status bns_backward_mixed(const bns_shape* shape, const bns_spec* spec, uint64_t seed,
                              int32_t n_v, float mix_beta,
                              const void* x, const void* dy, const float* gamma,
                              const float* save_mean, const float* save_invstd, const float* save_mean_parts,
                              void* dx, float* dgamma, float* dbeta,
                              void* workspace, size_t workspace_bytes, void* stream);

/* Inference-mode normalisation (App. D): the statistics are the recorded moving averages of Eq. 8,
 *   y = gamma * (x - running_mean) / sqrt(running_var + eps) + beta        for all points.
 * in: x, gamma, beta, running_mean, running_var.  out: y. */
bns_status bns_inference(const bns_shape* shape, const void* x, const float* gamma, const float* beta,
                         const float* running_mean, const float* running_var, float eps, void* y, void* stream);

/* Weight of the new statistics in Eq. 8 at training iteration `iteration` (counted from 1): 1 at the first
 * iteration, where the moving average starts as a copy of the statistics, alpha afterwards.  The value to
 * pass as `momentum` to bns_forward / bns_forward_mixed.  HOST function, no device is touched; iteration 0
 * is treated as the first.  (Appendix D reports a larger alpha than the customary 0.1 to work better for
 * the noisier sampled statistics, so alpha is the caller's choice.) */
float bns_moving_average_weight(uint64_t iteration, float alpha);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16) with 128-bit accesses:
 * the "achievable bandwidth" yardstick that the benchmark reports beside the BN kernels,
 * and the known-size kernel that hardware traffic counters are calibrated against. */
bns_status bns_copy_reference(void* dst, const void* src, size_t bytes, void* stream);

/* Process-wide overrides of launch choices, for benchmarking and tests; value 0 restores the
 * automatic choice.  name: HOST string.  Returns BNS_EINVAL for an unknown name or a value out of range.
 *   "path"           1: only the streaming kernels (statistics / normalise / reduce / dx, several
 *                    launches per direction); 2: only the fused single-launch kernels, which keep a
 *                    channel in registers between its reduction and its element-wise pass
 *                    (BNS_EUNSUPPORTED if a channel does not fit or the layout is N x H x W x C, which has
 *                    none); 0: whichever is faster for the shape
 *   "fused_variant"  1..7: block size / registers-per-thread variant of the fused kernels
 *   "fused_pipe"     the backward kernel that holds two channels per block, loading the next one while the
 *                    sums of the current one are exchanged: 1..6 that (block size, vectors) variant whatever
 *                    the shape, 16 never; 0: when the launch has three or more rounds (tensors below 4 GiB)
 *   "fused_team"     blocks that share a channel in that kernel, if they can hold it    (1..128)
 *   "fused_coop"     1: launch the fused kernels with hipLaunchCooperativeKernel
 *   "fused_patch_mask"  Feature Sampling forward: by default, when one block holds a channel, the statistics of
 *                    the patch come from the vectors already in registers, under a column mask (built for the
 *                    two largest variants and rows that are a whole number of vectors); 1: also when several
 *                    blocks share a channel; 2: the patch elements are always read on their own, ahead of
 *                    the vectors
 *   "fused_keep_x"   the fused backward kernel keeps x in registers beside dy instead of reading it again
 *                    on S: 1 always, 2 never; 0: when S is the whole tensor or a patch of every plane
 *   "split_statistics"  1: the streaming forward statistics always run as partial sums + finalize
 *                    (by default one 1024-thread block per channel does both when a channel has few
 *                    sampled points)
 *   "splits_stats"   blocks per channel in the statistics reduction (implies split_statistics) (1..64)
 *   "splits_reduce"  blocks per channel in the backward reduction                (1..64)
 *   "channel_group"  the streaming path walks the channels in groups of this many, every stage on
 *                    one group before the next                                   (1..C)
 *   "nhwc_blocks"    blocks that an N x H x W x C reduction launch aims for      (1..8192)
 *   "nhwc_ew_rows"   rows per thread in the N x H x W x C element-wise kernels   (1..2^20)
 *   "nhwc_split_dx"  1: the N x H x W x C backward writes dx on the rows outside S from its reduction kernel (Eq. 6
 *                    needs no sum there) and the rows of S from a kernel of their own; by default (and with 2)
 *                    the reduction is followed by one dx kernel over all rows, which is faster on this device
 *   "cache_reuse"    streaming kernels: a first pass (statistics; the sums of Eq. 5) loads what the pass after it
 *                    (Eq. 1; Eq. 6) reads again without the non-temporal hint, so that it stays in the device's
 *                    memory-side cache: 1 all of it, 2 none; 0: as much as fits there (224 MB).  Results do not
 *                    depend on it.
 *   "nhwc_small"     2: small N x H x W x C tensors also take the streaming kernels (by default one launch
 *                    per direction does everything when a thread would walk at most 16 rows)
 *   "norm_unroll", "dx_unroll", "reduce_unroll"   128-bit accesses per thread    (1, 2, 4)
 *   "norm_nt", "dx_nt"   non-temporal access mask + 1: bit 0 loads, bit 1 stores
 *   "reduce_nt"      the same for the backward reduction: bit 0 loads of x, bit 1 loads of dy, for the channels
 *                    that "cache_reuse" keeps (the others are loaded non-temporally)
 * Two more exist for the library's own tests only; they make results wrong on purpose and a caller has no
 * use for them:
 *   "test_spin_limit"    polls a block of a fused kernel waits for a team-mate's sums before it gives up
 *                    (1..2^21, the default)
 *   "test_mute_exchange" 1: no block publishes its sums, so every such wait runs out -- the two together let
 *                    a test reach the give-up path (NaN sums, the kernel ends normally) from the host
 * The options are atomics: setting one while another thread launches work is defined (that call sees the old
 * or the new value), but the launch choices of calls in flight are then anyone's guess -- set them first.
 * Notes on the fused kernels: blocks of a team exchange partial sums through the workspace and wait
 * for each other with a bounded spin (the grid never exceeds what the device holds at once); they
 * are bit-reproducible like the streaming kernels, and they can be captured into a HIP graph like any other
 * launch (the stamps that tell one exchange from the next are counted in the workspace, on the device). */
bns_status bns_set_option(const char* name, int32_t value);
/* Current value of an option (as set, 0 = automatic); also, kept per calling thread,
 * "last_path_forward" / "last_path_backward": 1 if this thread's last bns_forward / bns_backward took the streaming kernels, 2 if the fused one, 3 if the
 * one-launch kernel for small N x H x W x C tensors, 4 (backward, N x H x W x C) the streaming kernels with dx split
 * between the reduction kernel and a kernel for the rows of S ("nhwc_split_dx"); "last_fused_backward": which fused backward kernel that was
 * (1 plain, 2 x kept in registers, 3 pipelined); "last_fused_forward": 2 if the fused forward kernel took the
 * statistics of a patch from the registers (see "fused_patch_mask"), else 1; "launch_count": kernels launched by the library since it was
 * loaded, modulo 2^31 (benchmarks report launches per call from its differences).
 * -1 for an unknown name. */
int32_t bns_get_option(const char* name);

#ifdef __cplusplus
}
#endif
#endif /* BNS_H */
