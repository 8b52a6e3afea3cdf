// Sampling-index generator shared by the host entry points and the kernels.
//
// Alg. 1 and Alg. 2 of the paper draw begin = randint(0, N - n_s) and
// (begin_h, begin_w) = (randint(0, H - h_s), randint(0, W - w_s)) once per layer and
// epoch; the paper names no generator.  Here the draw is a counter-based integer hash,
// so that host and device compute the same index from the same five integers and
// nothing has to be stored: three rounds of the SplitMix64 finaliser over
// (seed, layer_id | epoch, tag | channel); the top 32 bits are scaled to the number of
// outcomes with a multiply and shift.  Both ends of the range are reachable, because
// the algorithms' slices end at begin + n_s - 1 inclusive.  Integer arithmetic only.
#pragma once
#include <stdint.h>

#include "../../include/bns.h"

#if defined(__HIPCC__)
#define BNS_HD __host__ __device__ inline
#else
#define BNS_HD inline
#endif

namespace bns {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;
constexpr uint32_t kTagN = 1u, kTagH = 2u, kTagW = 3u;  // which coordinate is drawn
constexpr uint32_t kSharedChannel = 0xFFFFFFFFu;         // one index for the whole layer

BNS_HD uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Hash state after seed, layer and epoch have been absorbed; computed once per call.
BNS_HD uint64_t index_key(uint64_t seed, uint32_t layer_id, uint32_t epoch) {
    uint64_t h = mix64(seed + kGolden);
    return mix64(h ^ ((uint64_t(layer_id) << 32) | uint64_t(epoch)));
}

// randint(0, k) with both ends included.
BNS_HD int32_t draw(uint64_t key, uint32_t tag, uint32_t channel, int32_t k) {
    uint64_t h = mix64(key ^ ((uint64_t(tag) << 32) | uint64_t(channel)));
    return int32_t(((h >> 32) * uint64_t(uint32_t(k) + 1u)) >> 32);
}

// Everything a kernel needs to rebuild the box of any channel.
struct IndexParams {
    bns_box shared;       // the box when it does not depend on the channel
    uint64_t key;         // index_key(seed, layer, epoch)
    int32_t per_channel;  // FS with an independent patch location per channel
    int32_t k_h, k_w;     // H - patch_h, W - patch_w (largest legal begin)
};

BNS_HD bns_box box_of_channel(const IndexParams& p, int32_t c) {
    bns_box b = p.shared;
    if (p.per_channel) {
        b.h0 = draw(p.key, kTagH, uint32_t(c), p.k_h);
        b.w0 = draw(p.key, kTagW, uint32_t(c), p.k_w);
    }
    return b;
}

// Host side: shape and spec are already validated.
inline IndexParams make_index_params(const bns_shape& sh, const bns_spec& sp, uint64_t seed) {
    IndexParams p;
    p.key = index_key(seed, sp.layer_id, sp.epoch);
    p.per_channel = 0;
    p.k_h = p.k_w = 0;
    bns_box b = {0, sh.N, 0, sh.H, 0, sh.W};
    switch (sp.mode) {
        case BNS_NS:
        case BNS_VDN:
            b.n_cnt = sp.n_s;
            break;
        case BNS_BS:
            b.n_cnt = sp.n_s;
            b.n0 = draw(p.key, kTagN, kSharedChannel, sh.N - sp.n_s);
            break;
        case BNS_FS:
            b.h_cnt = sp.patch_h;
            b.w_cnt = sp.patch_w;
            p.k_h = sh.H - sp.patch_h;
            p.k_w = sh.W - sp.patch_w;
            if (sp.fs_per_channel) {
                p.per_channel = 1;
            } else {
                b.h0 = draw(p.key, kTagH, kSharedChannel, p.k_h);
                b.w0 = draw(p.key, kTagW, kSharedChannel, p.k_w);
            }
            break;
        default:
            break;
    }
    p.shared = b;
    return p;
}

// "VDN + sampling" (Eq. 4): the first n_v samples are virtual, and the sampling strategy of
// `sp` is applied to the N - n_v real samples behind them (Alg. 1 / Alg. 2 on the real part of
// the batch, sample indices shifted by n_v).  Returns the index of the sampled REAL set.
inline IndexParams make_index_params_mixed(const bns_shape& sh, const bns_spec& sp, uint64_t seed, int32_t n_v) {
    bns_shape real = sh;
    real.N = sh.N - n_v;
    IndexParams p = make_index_params(real, sp, seed);
    p.shared.n0 += n_v;
    return p;
}

// The virtual set: samples 0 .. n_v-1, every row and column (Alg. 3).
inline IndexParams make_index_params_virtual(const bns_shape& sh, int32_t n_v) {
    IndexParams p;
    p.key = 0;
    p.per_channel = 0;
    p.k_h = p.k_w = 0;
    p.shared = bns_box{0, n_v, 0, sh.H, 0, sh.W};
    return p;
}

}  // namespace bns
