// HIP kernels of libbns for gfx950 (wave64).  All of them are bound by HBM traffic:
// a few flops per element moved, so no matrix cores; the work is to keep every access
// 128 bits wide and coalesced, to touch only the bytes the method needs, and to keep
// enough loads in flight.
//
// Data layout: N x C x H x W.  A channel is N planes of HW contiguous elements, one per
// sample, (C * HW) elements apart.  Within one sample the planes of consecutive channels
// are adjacent, so a channel range [c0, c0 + cg) of one sample is ONE contiguous run of
// cg * HW elements: the element-wise kernels walk that run with flat 128-bit accesses and
// recover the channel of an access with one multiply-shift division.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "bns_device.hpp"
#include "bns_internal.hpp"

namespace bns {

// ===========================================================================
// Forward statistics over the location set S (Eq. 3)
// ===========================================================================
// Sums are taken of (x - pivot), pivot = the first sampled element of the channel, so
// that Var = E[d^2] - E[d]^2 does not cancel when |mean| >> std.

// S made of whole planes (FULL, NS, BS, VDN) with HW a multiple of V.
// grid.x = cg * splits; block (c, k) reduces vectors [k * per_block, (k + 1) * per_block)
// of the n_cnt * HW / V vectors of channel c.
// KEEP: the sampled planes fit the memory-side cache, and the normalization pass that follows reads them again:
// plain loads leave them there, non-temporal ones (faster from memory) do not.
template <typename T, int V, bool KEEP>
__global__ __launch_bounds__(kBlock) void stats_partial_planes_kernel(
    const T* __restrict__ x, Partial* __restrict__ partial, IndexParams ip, int C, int HW,
    FastDiv hwv_div, int c0, int splits, uint32_t per_block) {
    __shared__ float lds[2 * (kBlock / kWave)];
    const int cl = blockIdx.x / splits;
    const int k = blockIdx.x - cl * splits;
    const int c = c0 + cl;
    const bns_box b = ip.shared;                                   // planes: never per-channel
    const uint32_t hwv = hwv_div.d;
    const uint32_t tot = uint32_t(b.n_cnt) * hwv;
    const uint32_t j0 = uint32_t(k) * per_block;
    const uint32_t j1 = min(j0 + per_block, tot);
    const size_t nstride = size_t(C) * HW;
    const T* base = x + (size_t(b.n0) * C + c) * HW;                // plane (n0, c)
    const float pivot = load_scalar<T>(base);

    float s1[2] = {0.f, 0.f}, s2[2] = {0.f, 0.f};
    uint32_t j = j0 + threadIdx.x;
    for (; j + 3u * kBlock < j1; j += 4u * kBlock) {
        Vec<T, V> v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t ju = j + u * kBlock;
            const uint32_t n = fdiv(ju, hwv_div);
            const T* p = base + n * nstride + size_t(ju - n * hwv) * V;
            if (KEEP) v[u].load(p); else v[u].load_nt(p);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const float dlt = v[u].f[i] - pivot;
                s1[u & 1] += dlt;
                s2[u & 1] = fmaf(dlt, dlt, s2[u & 1]);
            }
    }
    for (; j < j1; j += kBlock) {
        const uint32_t n = fdiv(j, hwv_div);
        Vec<T, V> v;
        v.load(base + n * nstride + size_t(j - n * hwv) * V);
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float dlt = v.f[i] - pivot;
            s1[0] += dlt;
            s2[0] = fmaf(dlt, dlt, s2[0]);
        }
    }
    float a = s1[0] + s1[1], q = s2[0] + s2[1];
    block_sum2(a, q, lds);
    if (threadIdx.x == 0) partial[size_t(c) * splits + k] = Partial{a, q};
}

// S a rectangular patch of every sampled plane (FS), or planes whose size is not a
// multiple of the vector width.  Scalar accesses: patch rows are short and unaligned.
// Element j of the n_cnt * h_cnt * w_cnt sampled points -> (n, ph, pw) by two divisions.
template <typename T>
__global__ __launch_bounds__(kBlock) void stats_partial_patch_kernel(
    const T* __restrict__ x, Partial* __restrict__ partial, IndexParams ip, int C, int W, int HW,
    FastDiv patch_div, FastDiv pw_div, int c0, int splits, uint32_t per_block) {
    __shared__ float lds[2 * (kBlock / kWave)];
    const int cl = blockIdx.x / splits;
    const int k = blockIdx.x - cl * splits;
    const int c = c0 + cl;
    const bns_box b = box_of_channel(ip, c);
    const uint32_t tot = uint32_t(b.n_cnt) * patch_div.d;
    const uint32_t j0 = uint32_t(k) * per_block;
    const uint32_t j1 = min(j0 + per_block, tot);
    const size_t nstride = size_t(C) * HW;
    const T* base = x + (size_t(b.n0) * C + c) * HW + size_t(b.h0) * W + b.w0;   // first sampled element
    const float pivot = load_scalar<T>(base);

    auto at = [&](uint32_t j) {
        const uint32_t n = fdiv(j, patch_div);
        const uint32_t r = j - n * patch_div.d;
        const uint32_t ph = fdiv(r, pw_div);
        const uint32_t pw = r - ph * pw_div.d;
        return load_scalar<T>(base + n * nstride + size_t(ph) * W + pw);
    };
    float s1 = 0.f, s2 = 0.f;
    uint32_t j = j0 + threadIdx.x;
    for (; j + 3u * kBlock < j1; j += 4u * kBlock) {        // four independent loads in flight
        const float v0 = at(j), v1 = at(j + kBlock), v2 = at(j + 2u * kBlock), v3 = at(j + 3u * kBlock);
        const float d0 = v0 - pivot, d1 = v1 - pivot, d2 = v2 - pivot, d3 = v3 - pivot;
        s1 += (d0 + d1) + (d2 + d3);
        s2 = fmaf(d0, d0, fmaf(d1, d1, fmaf(d2, d2, fmaf(d3, d3, s2))));
    }
    for (; j < j1; j += kBlock) {
        const float dlt = at(j) - pivot;
        s1 += dlt;
        s2 = fmaf(dlt, dlt, s2);
    }
    block_sum2(s1, s2, lds);
    if (threadIdx.x == 0) partial[size_t(c) * splits + k] = Partial{s1, s2};
}

// Few sampled points per channel (Batch Sampling or Feature Sampling at the paper's ratios): ONE
// block of 1024 threads per channel reduces all of them and applies Eq. 3 and Eq. 8 itself, so
// the statistics need a single launch and no hand-over between blocks.
// PLANES: S made of whole planes and HW a multiple of V (128-bit accesses); else scalar patch walk.
constexpr int kOneBlock = 1024;
template <typename T, int V, bool PLANES>
__global__ __launch_bounds__(kOneBlock) void stats_one_block_kernel(
    const T* __restrict__ x, IndexParams ip, int C, int W, int HW, FastDiv hwv_div, FastDiv patch_div, FastDiv pw_div,
    int c0, float eps, float momentum, float* __restrict__ save_mean, float* __restrict__ save_invstd,
    float* __restrict__ running_mean, float* __restrict__ running_var) {
    __shared__ float lds[2 * (kOneBlock / kWave)];
    const int c = c0 + blockIdx.x;
    const bns_box b = box_of_channel(ip, c);
    const size_t nstride = size_t(C) * HW;
    const T* base = x + (size_t(b.n0) * C + c) * HW + size_t(b.h0) * W + b.w0;   // first sampled element
    const float pivot = load_scalar<T>(base);
    float s1 = 0.f, s2 = 0.f;
    if (PLANES) {
        const uint32_t hwv = hwv_div.d;
        const uint32_t tot = uint32_t(b.n_cnt) * hwv;
        constexpr int U = 8;                                   // all of a thread's loads in flight at once
        for (uint32_t j0 = threadIdx.x; j0 < tot; j0 += U * kOneBlock) {
            Vec<T, V> v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t j = j0 + u * kOneBlock;
                if (j < tot) {
                    const uint32_t n = fdiv(j, hwv_div);
                    v[u].load(base + n * nstride + size_t(j - n * hwv) * V);   // (few points, read again by Eq. 1: plain)
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t j = j0 + u * kOneBlock;
                if (j < tot) {
#pragma unroll
                    for (int i = 0; i < V; ++i) {
                        const float dlt = v[u].f[i] - pivot;
                        s1 += dlt;
                        s2 = fmaf(dlt, dlt, s2);
                    }
                }
            }
        }
    } else {
        const uint32_t tot = uint32_t(b.n_cnt) * patch_div.d;
        constexpr int U = 16;                                  // scalar loads: one round trip for all of them
        for (uint32_t j0 = threadIdx.x; j0 < tot; j0 += U * kOneBlock) {
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t j = j0 + u * kOneBlock;
                if (j < tot) {
                    const uint32_t n = fdiv(j, patch_div);
                    const uint32_t r = j - n * patch_div.d;
                    const uint32_t ph = fdiv(r, pw_div);
                    v[u] = load_scalar<T>(base + n * nstride + size_t(ph) * W + (r - ph * pw_div.d));
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (j0 + u * kOneBlock < tot) {
                    const float dlt = v[u] - pivot;
                    s1 += dlt;
                    s2 = fmaf(dlt, dlt, s2);
                }
            }
        }
    }
    block_sum2<kOneBlock>(s1, s2, lds);
    if (threadIdx.x != 0) return;
    const double s = double(b.n_cnt) * double(b.h_cnt) * double(b.w_cnt);
    const double m1 = double(s1) / s;
    const double mean = double(pivot) + m1;
    double var = double(s2) / s - m1 * m1;
    if (var < 0.0) var = 0.0;
    save_mean[c] = float(mean);
    save_invstd[c] = float(1.0 / sqrt(var + double(eps)));
    const double a = double(momentum);
    if (running_mean) running_mean[c] = float((1.0 - a) * double(running_mean[c]) + a * mean);
    if (running_var) running_var[c] = float((1.0 - a) * double(running_var[c]) + a * var);
}

// One wave per channel: lane k holds split k, fp64 butterfly (a fixed pattern, so the
// rounding order never changes), then lane 0 applies Eq. 3 and Eq. 8.  splits <= 64.
template <typename T>
__global__ __launch_bounds__(kBlock) void stats_finalize_kernel(
    const T* __restrict__ x, const Partial* __restrict__ partial, IndexParams ip, int C, int W, int HW,
    int splits, int c0, int cg, float eps, float momentum, float* __restrict__ save_mean,
    float* __restrict__ save_invstd, float* __restrict__ running_mean, float* __restrict__ running_var) {
    const int lane = threadIdx.x % kWave;
    const int cl = blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (cl >= cg) return;                                           // whole wave leaves together
    const int c = c0 + cl;
    double s1 = 0.0, s2 = 0.0;
    if (lane < splits) {
        const Partial p = partial[size_t(c) * splits + lane];
        s1 = double(p.a);
        s2 = double(p.b);
    }
    // loads that lane 0 needs, issued before the shuffles
    const bns_box b = box_of_channel(ip, c);
    double pivot = 0.0, rm = 0.0, rv = 0.0;
    if (lane == 0) {
        pivot = load_scalar<T>(x + (size_t(b.n0) * C + c) * HW + size_t(b.h0) * W + b.w0);
        if (running_mean) rm = double(running_mean[c]);
        if (running_var) rv = double(running_var[c]);
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if (lane != 0) return;
    const double s = double(b.n_cnt) * double(b.h_cnt) * double(b.w_cnt);
    const double m1 = s1 / s;
    const double mean = pivot + m1;
    double var = s2 / s - m1 * m1;
    if (var < 0.0) var = 0.0;
    save_mean[c] = float(mean);
    save_invstd[c] = float(1.0 / sqrt(var + double(eps)));
    const double a = double(momentum);
    if (running_mean) running_mean[c] = float((1.0 - a) * rm + a * mean);
    if (running_var) running_var[c] = float((1.0 - a) * rv + a * var);
}

// "VDN + sampling" (Eq. 4): one wave per channel combines the partial sums of the sampled real
// set and of the virtual set, each into its own E and Var (Eq. 3), and blends them.
template <typename T>
__global__ __launch_bounds__(kBlock) void stats_finalize_mixed_kernel(
    const T* __restrict__ x, const Partial* __restrict__ partial_s, int splits_s,
    const Partial* __restrict__ partial_v, int splits_v, IndexParams ip_s, IndexParams ip_v, int C, int W, int HW,
    float mix_beta, float eps, float momentum, float* __restrict__ save_mean, float* __restrict__ save_invstd,
    float* __restrict__ mean_parts, float* __restrict__ running_mean, float* __restrict__ running_var) {
    const int lane = threadIdx.x % kWave;
    const int c = blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (c >= C) return;
    double a1 = 0.0, a2 = 0.0, v1 = 0.0, v2 = 0.0;
    if (lane < splits_s) {
        const Partial p = partial_s[size_t(c) * splits_s + lane];
        a1 = double(p.a);
        a2 = double(p.b);
    }
    if (lane < splits_v) {
        const Partial p = partial_v[size_t(c) * splits_v + lane];
        v1 = double(p.a);
        v2 = double(p.b);
    }
    const bns_box bs = box_of_channel(ip_s, c);
    const bns_box bv = ip_v.shared;
    double piv_s = 0.0, piv_v = 0.0, rm = 0.0, rv = 0.0;
    if (lane == 0) {
        piv_s = load_scalar<T>(x + (size_t(bs.n0) * C + c) * HW + size_t(bs.h0) * W + bs.w0);
        piv_v = load_scalar<T>(x + size_t(c) * HW);
        if (running_mean) rm = double(running_mean[c]);
        if (running_var) rv = double(running_var[c]);
    }
    a1 = wave_sum(a1);
    a2 = wave_sum(a2);
    v1 = wave_sum(v1);
    v2 = wave_sum(v2);
    if (lane != 0) return;
    const double ss = double(bs.n_cnt) * double(bs.h_cnt) * double(bs.w_cnt);
    const double sv = double(bv.n_cnt) * double(bv.h_cnt) * double(bv.w_cnt);
    const double ms = a1 / ss, mv = v1 / sv;
    const double e_s = piv_s + ms, e_v = piv_v + mv;
    double var_s = a2 / ss - ms * ms, var_v = v2 / sv - mv * mv;
    if (var_s < 0.0) var_s = 0.0;
    if (var_v < 0.0) var_v = 0.0;
    const double bm = double(mix_beta);
    const double mean = bm * e_v + (1.0 - bm) * e_s;            // Eq. 4, X = E
    const double var = bm * var_v + (1.0 - bm) * var_s;         // Eq. 4, X = Var
    save_mean[c] = float(mean);
    save_invstd[c] = float(1.0 / sqrt(var + double(eps)));
    mean_parts[c] = float(e_v);
    mean_parts[C + c] = float(e_s);
    const double al = double(momentum);
    if (running_mean) running_mean[c] = float((1.0 - al) * rm + al * mean);
    if (running_var) running_var[c] = float((1.0 - al) * rv + al * var);
}

// ===========================================================================
// Forward normalise + affine over every element (Eq. 1)
// ===========================================================================
// grid = (ceil(cg * HW / V / (kBlock * U)), N).  Block (bx, n) handles kBlock * U
// consecutive vectors of the contiguous run [c0, c0 + cg) x HW of sample n.
template <typename T, int V, int U, int NT>
__global__ __launch_bounds__(kBlock) void normalize_kernel(
    const T* __restrict__ x, T* __restrict__ y, const float* __restrict__ gamma,
    const float* __restrict__ beta, const float* __restrict__ mean, const float* __restrict__ invstd,
    int C, int HW, FastDiv hwv_div, int c0, uint32_t run_vectors, float var_eps) {
    // var_eps >= 0: `invstd` holds variances (inference from the moving averages, App. D) and
    // 1 / sqrt(var + var_eps) is taken here; var_eps < 0: it holds inverse standard deviations.
    const size_t run0 = (size_t(blockIdx.y) * C + c0) * HW;
    const T* xr = x + run0;
    T* yr = y + run0;
    const uint32_t v0 = blockIdx.x * uint32_t(kBlock * U) + threadIdx.x;

    Vec<T, V> v[U];
    float mu[U], sc[U], sh[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t vi = v0 + u * kBlock;
        if (vi < run_vectors) {
            if (NT & 1) v[u].load_nt(xr + size_t(vi) * V); else v[u].load(xr + size_t(vi) * V);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t vi = v0 + u * kBlock;
        if (vi < run_vectors) {
            const int c = c0 + int(fdiv(vi, hwv_div));
            mu[u] = mean[c];
            const float r = var_eps >= 0.f ? 1.0f / sqrtf(invstd[c] + var_eps) : invstd[c];
            sc[u] = gamma[c] * r;
            sh[u] = beta[c];
        }
    }
    // (x - mean) first: exact when x is close to the mean, where folding the mean into the
    // shift (x * sc + (beta - mean * sc)) would cancel.
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t vi = v0 + u * kBlock;
        if (vi < run_vectors) {
#pragma unroll
            for (int i = 0; i < V; ++i) v[u].f[i] = fmaf(v[u].f[i] - mu[u], sc[u], sh[u]);
            if (NT & 2) v[u].store_nt(yr + size_t(vi) * V); else v[u].store(yr + size_t(vi) * V);
        }
    }
}

// ===========================================================================
// Backward reductions over all m points (Eq. 5): sum dy, sum dy * (x - mean)
// ===========================================================================
// grid.x = cg * splits, block (c, k) as in stats_partial_planes_kernel with S = everything.
// NT: bit 0 non-temporal loads of x, bit 1 of dy.  What the dx pass reads again (dy; x too when S is everything)
// is loaded plainly when it fits the memory-side cache, so that the dx pass finds it there.
template <typename T, int V, int U, int NT>
__global__ __launch_bounds__(kBlock) void reduce_partial_kernel(
    const T* __restrict__ x, const T* __restrict__ dy, const float* __restrict__ mean,
    Partial* __restrict__ partial, int C, int HW, FastDiv hwv_div, int c0, int splits, uint32_t per_block,
    uint32_t tot, int keep_channels) {
    __shared__ float lds[2 * (kBlock / kWave)];
    const int cl = blockIdx.x / splits;       // consecutive blocks: consecutive ranges of the same channel
    const int k = blockIdx.x - cl * splits;
    const int c = c0 + cl;
    const uint32_t hwv = hwv_div.d;
    const uint32_t j0 = uint32_t(k) * per_block;
    const uint32_t j1 = min(j0 + per_block, tot);
    const size_t nstride = size_t(C) * HW;
    const size_t cbase = size_t(c) * HW;
    const float mu = mean[c];

    float s1[U], s2[U];
#pragma unroll
    for (int u = 0; u < U; ++u) s1[u] = s2[u] = 0.f;
    auto walk = [&](auto mask) {
        constexpr int M = decltype(mask)::value;
        uint32_t j = j0 + threadIdx.x;
        for (; j + uint32_t(U - 1) * kBlock < j1; j += uint32_t(U) * kBlock) {
            Vec<T, V> g[U], v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t ju = j + u * kBlock;
                const uint32_t n = fdiv(ju, hwv_div);
                const size_t off = cbase + n * nstride + size_t(ju - n * hwv) * V;
                if (M & 2) g[u].load_nt(dy + off); else g[u].load(dy + off);
                if (M & 1) v[u].load_nt(x + off); else v[u].load(x + off);
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    s1[u] += g[u].f[i];
                    s2[u] = fmaf(g[u].f[i], v[u].f[i] - mu, s2[u]);
                }
        }
        for (; j < j1; j += kBlock) {
            const uint32_t n = fdiv(j, hwv_div);
            const size_t off = cbase + n * nstride + size_t(j - n * hwv) * V;
            Vec<T, V> g, v;
            g.load(dy + off);
            v.load(x + off);
#pragma unroll
            for (int i = 0; i < V; ++i) {
                s1[0] += g.f[i];
                s2[0] = fmaf(g.f[i], v.f[i] - mu, s2[0]);
            }
        }
    };
    // the channels whose dy (and x) fit the memory-side cache take the loads that the mask asks for, the others
    // the non-temporal ones (the same for the whole block)
    if (NT == 3 || cl < keep_channels) walk(std::integral_constant<int, NT>());
    else walk(std::integral_constant<int, 3>());
    float a = s1[0], q = s2[0];
#pragma unroll
    for (int u = 1; u < U; ++u) {
        a += s1[u];
        q += s2[u];
    }
    block_sum2(a, q, lds);
    if (threadIdx.x == 0) partial[size_t(c) * splits + k] = Partial{a, q};
}

__global__ __launch_bounds__(kBlock) void reduce_finalize_kernel(
    const Partial* __restrict__ partial, int splits, int c0, int cg, const float* __restrict__ invstd,
    float* __restrict__ dgamma, float* __restrict__ dbeta) {
    const int lane = threadIdx.x % kWave;
    const int cl = blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (cl >= cg) return;
    const int c = c0 + cl;
    double s1 = 0.0, s2 = 0.0;
    if (lane < splits) {
        const Partial p = partial[size_t(c) * splits + lane];
        s1 = double(p.a);
        s2 = double(p.b);
    }
    const float r = lane == 0 ? invstd[c] : 0.f;
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if (lane != 0) return;
    dbeta[c] = float(s1);
    dgamma[c] = float(s2 * double(r));
}

// ===========================================================================
// Backward dx over every element (Eq. 6)
// ===========================================================================
// Same walk as normalize_kernel.  dx = a * dy everywhere (a = gamma * invstd); the
// 1/s terms of Eq. 6 are subtracted only where the element lies in S, and x is loaded
// only by accesses that intersect S.
template <typename T, int V, int U, int NT>
__global__ __launch_bounds__(kBlock) void dx_kernel(
    const T* __restrict__ x, const T* __restrict__ dy, T* __restrict__ dx, const float* __restrict__ gamma,
    const float* __restrict__ mean, const float* __restrict__ invstd, const float* __restrict__ dgamma,
    const float* __restrict__ dbeta, IndexParams ip, int C, int W, int HW, FastDiv hwv_div, FastDiv w_div,
    int c0, uint32_t run_vectors, DxSets sets) {
    const int n = blockIdx.y;
    const bool virt = n < sets.n_v;                 // sample of the virtual set (Eq. 4); block-uniform
    const float wgt = virt ? sets.w_v : sets.w_s;
    const float* __restrict__ centre = virt ? sets.centre_v : sets.centre_s;
    const size_t run0 = (size_t(n) * C + c0) * HW;
    const T* xr = x + run0;
    const T* gr = dy + run0;
    T* dr = dx + run0;
    const uint32_t v0 = blockIdx.x * uint32_t(kBlock * U) + threadIdx.x;
    const uint32_t hwv = hwv_div.d;

    Vec<T, V> g[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t vi = v0 + u * kBlock;
        if (vi < run_vectors) {
            if (NT & 1) g[u].load_nt(gr + size_t(vi) * V); else g[u].load(gr + size_t(vi) * V);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t vi = v0 + u * kBlock;
        if (vi >= run_vectors) continue;
        const uint32_t cl = fdiv(vi, hwv_div);
        const int c = c0 + int(cl);
        const uint32_t e0 = (vi - cl * hwv) * V;                  // first element, within its plane
        const bns_box b = virt ? bns_box{0, sets.n_v, 0, HW / W, 0, W} : box_of_channel(ip, c);
        const float r = invstd[c];
        const float a = gamma[c] * r;
        // rows [h0, h0 + h_cnt) of the plane are the elements [h0 * W, (h0 + h_cnt) * W)
        const bool touches = n >= b.n0 && n < b.n0 + b.n_cnt && e0 + V > uint32_t(b.h0) * W &&
                             e0 < uint32_t(b.h0 + b.h_cnt) * W;
        if (touches) {
            Vec<T, V> xv;
            if (NT & 1) xv.load_nt(xr + size_t(vi) * V); else xv.load(xr + size_t(vi) * V);
            const float mu = centre[c];
            const float k1 = a * wgt * dbeta[c];
            const float k2 = a * wgt * dgamma[c] * r;
            uint32_t h = fdiv(e0, w_div);
            uint32_t w = e0 - h * uint32_t(W);
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const bool in = h >= uint32_t(b.h0) && h < uint32_t(b.h0 + b.h_cnt) &&
                                w >= uint32_t(b.w0) && w < uint32_t(b.w0 + b.w_cnt);
                const float corr = in ? fmaf(k2, xv.f[i] - mu, k1) : 0.f;
                g[u].f[i] = fmaf(a, g[u].f[i], -corr);
                if (++w == uint32_t(W)) {
                    w = 0;
                    ++h;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < V; ++i) g[u].f[i] *= a;
        }
        if (NT & 2) g[u].store_nt(dr + size_t(vi) * V); else g[u].store(dr + size_t(vi) * V);
    }
}

// ===========================================================================
// Utilities
// ===========================================================================
__global__ __launch_bounds__(kBlock) void index_boxes_kernel(IndexParams ip, int C, bns_box* __restrict__ boxes) {
    const int c = blockIdx.x * kBlock + threadIdx.x;
    if (c < C) boxes[c] = box_of_channel(ip, c);
}

__global__ __launch_bounds__(kBlock) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                      size_t n16) {
    const size_t i0 = size_t(blockIdx.x) * (kBlock * 4) + threadIdx.x;
    if (i0 + 3 * kBlock < n16) {
        const uint4 a = src[i0], b = src[i0 + kBlock], c = src[i0 + 2 * kBlock], d = src[i0 + 3 * kBlock];
        dst[i0] = a;
        dst[i0 + kBlock] = b;
        dst[i0 + 2 * kBlock] = c;
        dst[i0 + 3 * kBlock] = d;
    } else {
        for (size_t i = i0; i < n16; i += kBlock) dst[i] = src[i];
    }
}

// ===========================================================================
// Launchers
// ===========================================================================
namespace {

inline uint32_t ceil_div(uint32_t a, uint32_t b) { return (a + b - 1) / b; }

// Calls f(T tag, integral_constant<V>) for the storage type and vector width of `d`.
template <int V>
struct VecTag {
    static constexpr int value = V;
};

template <int I>
struct IC {
    static constexpr int value = I;
};

// Calls f(IC<U>, IC<NT>) for an unroll factor in {1, 2, 4} and a non-temporal mask in 0..3.
template <typename F>
hipError_t dispatch_unroll_nt(int U, int NT, F&& f) {
    switch ((U == 1 ? 0 : U == 2 ? 1 : 2) * 4 + (NT & 3)) {
        case 0: return f(IC<1>(), IC<0>());
        case 1: return f(IC<1>(), IC<1>());
        case 2: return f(IC<1>(), IC<2>());
        case 3: return f(IC<1>(), IC<3>());
        case 4: return f(IC<2>(), IC<0>());
        case 5: return f(IC<2>(), IC<1>());
        case 6: return f(IC<2>(), IC<2>());
        case 7: return f(IC<2>(), IC<3>());
        case 8: return f(IC<4>(), IC<0>());
        case 9: return f(IC<4>(), IC<1>());
        case 10: return f(IC<4>(), IC<2>());
        default: return f(IC<4>(), IC<3>());
    }
}

template <typename F>
hipError_t dispatch(const Dims& d, F&& f) {
    if (d.dtype == BNS_F32) {
        if (d.vec == 4) return f(float(), VecTag<4>());
        return f(float(), VecTag<1>());
    }
    if (d.vec == 8) return f(bf16_t(), VecTag<8>());
    if (d.vec == 4) return f(bf16_t(), VecTag<4>());
    return f(bf16_t(), VecTag<1>());
}

}  // namespace

Tuning g_tuning;

int auto_splits(int cg, uint32_t vectors_per_channel) {
    // Aim for >= 2048 blocks (8 per CU on 256 CUs) but keep >= 4 accesses per thread.
    uint32_t want = ceil_div(2048u, uint32_t(cg));
    uint32_t cap = vectors_per_channel / (4u * kBlock);
    if (cap < 1u) cap = 1u;
    uint32_t s = want < cap ? want : cap;
    if (s < 1u) s = 1u;
    if (s > uint32_t(kMaxSplits)) s = kMaxSplits;
    return int(s);
}

hipError_t launch_stats_partial(const Dims& d, const IndexParams& ip, const void* x, Partial* partial,
                                int splits, int c0, int cg, hipStream_t st) {
    const bns_box& b = ip.shared;
    const bool planes = !ip.per_channel && b.h_cnt == d.H && b.w_cnt == d.W && d.vec > 1;
    const dim3 grid(uint32_t(cg) * uint32_t(splits));
    if (planes) {
        return dispatch(d, [&](auto t, auto vt) {
            using T = decltype(t);
            constexpr int V = decltype(vt)::value;
            const uint32_t hwv = uint32_t(d.HW / V);
            const uint32_t tot = uint32_t(b.n_cnt) * hwv;
            const uint32_t per_block = ceil_div(tot, uint32_t(splits));
            if (keep_for_next_pass(size_t(tot) * V * sizeof(T) * size_t(cg)))
                BNS_LAUNCH((stats_partial_planes_kernel<T, V, true>), grid, dim3(kBlock), 0, st,
                           static_cast<const T*>(x), partial, ip, d.C, d.HW, make_fastdiv(hwv), c0, splits,
                           per_block);
            else
                BNS_LAUNCH((stats_partial_planes_kernel<T, V, false>), grid, dim3(kBlock), 0, st,
                           static_cast<const T*>(x), partial, ip, d.C, d.HW, make_fastdiv(hwv), c0, splits,
                           per_block);
            return hipGetLastError();
        });
    }
    const uint32_t patch = uint32_t(b.h_cnt) * uint32_t(b.w_cnt);
    const uint32_t tot = uint32_t(b.n_cnt) * patch;
    const uint32_t per_block = ceil_div(tot, uint32_t(splits));
    if (d.dtype == BNS_F32)
        BNS_LAUNCH((stats_partial_patch_kernel<float>), grid, dim3(kBlock), 0, st,
                   static_cast<const float*>(x), partial, ip, d.C, d.W, d.HW, make_fastdiv(patch),
                   make_fastdiv(uint32_t(b.w_cnt)), c0, splits, per_block);
    else
        BNS_LAUNCH((stats_partial_patch_kernel<bf16_t>), grid, dim3(kBlock), 0, st,
                   static_cast<const bf16_t*>(x), partial, ip, d.C, d.W, d.HW, make_fastdiv(patch),
                   make_fastdiv(uint32_t(b.w_cnt)), c0, splits, per_block);
    return hipGetLastError();
}

// Statistics in one launch, one block per channel; false if the channel has too many sampled
// points for that (the caller then uses partial sums + finalize).
bool launch_stats_one_block(const Dims& d, const IndexParams& ip, const void* x, int c0, int cg, float eps,
                            float momentum, float* save_mean, float* save_invstd, float* running_mean,
                            float* running_var, hipStream_t st, hipError_t* err) {
    const bns_box& b = ip.shared;
    const bool planes = !ip.per_channel && b.h_cnt == d.H && b.w_cnt == d.W && d.vec > 1;
    const uint64_t pts = uint64_t(b.n_cnt) * b.h_cnt * b.w_cnt;
    const uint64_t accesses = planes ? pts / d.vec : pts;
    if (accesses > uint64_t(kOneBlock) * 16 || cg < 64) return false;     // <= 16 accesses per thread; enough blocks
    const uint32_t hwv = uint32_t(d.HW / d.vec);
    const uint32_t patch = uint32_t(b.h_cnt) * uint32_t(b.w_cnt);
    const dim3 grid{uint32_t(cg)}, blk{uint32_t(kOneBlock)};
    *err = dispatch(d, [&](auto t, auto vt) {
        using T = decltype(t);
        constexpr int V = decltype(vt)::value;
        if (planes)
            BNS_LAUNCH((stats_one_block_kernel<T, V, true>), grid, blk, 0, st, static_cast<const T*>(x), ip, d.C,
                       d.W, d.HW, make_fastdiv(hwv), make_fastdiv(patch), make_fastdiv(uint32_t(b.w_cnt)), c0,
                       eps, momentum, save_mean, save_invstd, running_mean, running_var);
        else
            BNS_LAUNCH((stats_one_block_kernel<T, V, false>), grid, blk, 0, st, static_cast<const T*>(x), ip,
                       d.C, d.W, d.HW, make_fastdiv(hwv), make_fastdiv(patch),
                       make_fastdiv(uint32_t(b.w_cnt)), c0, eps, momentum, save_mean, save_invstd, running_mean,
                       running_var);
        return hipGetLastError();
    });
    return true;
}

hipError_t launch_stats_finalize(const Dims& d, const IndexParams& ip, const void* x, const Partial* partial,
                                 int splits, int c0, int cg, float eps, float momentum, float* save_mean,
                                 float* save_invstd, float* running_mean, float* running_var, hipStream_t st) {
    const dim3 grid(ceil_div(uint32_t(cg), kBlock / kWave));
    if (d.dtype == BNS_F32)
        BNS_LAUNCH((stats_finalize_kernel<float>), grid, dim3(kBlock), 0, st,
                   static_cast<const float*>(x), partial, ip, d.C, d.W, d.HW, splits, c0, cg, eps, momentum,
                   save_mean, save_invstd, running_mean, running_var);
    else
        BNS_LAUNCH((stats_finalize_kernel<bf16_t>), grid, dim3(kBlock), 0, st,
                   static_cast<const bf16_t*>(x), partial, ip, d.C, d.W, d.HW, splits, c0, cg, eps, momentum,
                   save_mean, save_invstd, running_mean, running_var);
    return hipGetLastError();
}

hipError_t launch_stats_finalize_mixed(const Dims& d, const IndexParams& ip_s, const IndexParams& ip_v, const void* x,
                                       const Partial* partial_s, int splits_s, const Partial* partial_v,
                                       int splits_v, float mix_beta, float eps, float momentum, float* save_mean,
                                       float* save_invstd, float* mean_parts, float* running_mean,
                                       float* running_var, hipStream_t st) {
    const dim3 grid(ceil_div(uint32_t(d.C), kBlock / kWave));
    if (d.dtype == BNS_F32)
        BNS_LAUNCH((stats_finalize_mixed_kernel<float>), grid, dim3(kBlock), 0, st,
                   static_cast<const float*>(x), partial_s, splits_s, partial_v, splits_v, ip_s, ip_v, d.C, d.W,
                   d.HW, mix_beta, eps, momentum, save_mean, save_invstd, mean_parts, running_mean, running_var);
    else
        BNS_LAUNCH((stats_finalize_mixed_kernel<bf16_t>), grid, dim3(kBlock), 0, st,
                   static_cast<const bf16_t*>(x), partial_s, splits_s, partial_v, splits_v, ip_s, ip_v, d.C,
                   d.W, d.HW, mix_beta, eps, momentum, save_mean, save_invstd, mean_parts, running_mean,
                   running_var);
    return hipGetLastError();
}

hipError_t launch_normalize(const Dims& d, const void* x, const float* gamma, const float* beta,
                            const float* mean, const float* invstd, void* y, int c0, int cg, hipStream_t st,
                            float var_eps) {
    return dispatch(d, [&](auto t, auto vt) {
        using T = decltype(t);
        constexpr int V = decltype(vt)::value;
        return dispatch_unroll_nt(tuned(g_tuning.norm_unroll, d.dtype == BNS_F32 ? 1 : 2), tuned_nt(g_tuning.norm_nt, 3), [&](auto ut, auto nt) {
            constexpr int U = decltype(ut)::value;
            constexpr int NT = decltype(nt)::value;
            const uint32_t hwv = uint32_t(d.HW / V);
            const uint32_t run_vectors = uint32_t(cg) * hwv;
            const dim3 grid(ceil_div(run_vectors, kBlock * U), uint32_t(d.N));
            BNS_LAUNCH((normalize_kernel<T, V, U, NT>), grid, dim3(kBlock), 0, st, static_cast<const T*>(x),
                       static_cast<T*>(y), gamma, beta, mean, invstd, d.C, d.HW, make_fastdiv(hwv), c0,
                       run_vectors, var_eps);
            return hipGetLastError();
        });
    });
}

hipError_t launch_reduce_partial(const Dims& d, const void* x, const void* dy, const float* mean,
                                 Partial* partial, int splits, int c0, int cg, bool x_again, hipStream_t st) {
    // dy of as many channels as fit stays in the memory-side cache for the dx pass (x too if that pass reads most of
    // it again)
    const size_t per_channel = size_t(d.N) * d.HW * (d.dtype == BNS_F32 ? 4 : 2);
    const int reuse = g_tuning.cache_reuse;
    const bool both = x_again;
    const size_t fit = kKeepBytes / (per_channel * (both ? 2 : 1));
    const int keep_channels = reuse == 2 ? 0 : reuse == 1 ? cg : int(std::min<size_t>(size_t(cg), fit));
    const int keep = keep_channels == 0 ? 0 : both ? 2 : 1;
    return dispatch(d, [&](auto t, auto vt) {
        using T = decltype(t);
        constexpr int V = decltype(vt)::value;
        return dispatch_unroll_nt(tuned(g_tuning.reduce_unroll, 2), tuned_nt(g_tuning.reduce_nt, keep == 2 ? 0 : keep == 1 ? 1 : 3), [&](auto ut, auto nt) {
            constexpr int U = decltype(ut)::value;
            constexpr int NT = decltype(nt)::value;
            const uint32_t hwv = uint32_t(d.HW / V);
            const uint32_t tot = uint32_t(d.N) * hwv;
            const uint32_t per_block = ceil_div(tot, uint32_t(splits));
            const dim3 grid(uint32_t(cg) * uint32_t(splits));
            BNS_LAUNCH((reduce_partial_kernel<T, V, U, NT>), grid, dim3(kBlock), 0, st,
                       static_cast<const T*>(x), static_cast<const T*>(dy), mean, partial, d.C, d.HW,
                       make_fastdiv(hwv), c0, splits, per_block, tot, keep_channels);
            return hipGetLastError();
        });
    });
}

hipError_t launch_reduce_finalize(const Dims& d, const Partial* partial, int splits, int c0, int cg,
                                  const float* invstd, float* dgamma, float* dbeta, hipStream_t st) {
    (void)d;
    BNS_LAUNCH(reduce_finalize_kernel, dim3(ceil_div(uint32_t(cg), kBlock / kWave)), dim3(kBlock), 0, st, partial,
               splits, c0, cg, invstd, dgamma, dbeta);
    return hipGetLastError();
}

hipError_t launch_dx(const Dims& d, const IndexParams& ip, const void* x, const void* dy, const float* gamma,
                     const float* mean, const float* invstd, const float* dgamma, const float* dbeta, void* dx,
                     int c0, int cg, hipStream_t st, const DxSets* mixed) {
    const bns_box& b = ip.shared;
    const double s = double(b.n_cnt) * double(b.h_cnt) * double(b.w_cnt);
    DxSets sets;
    if (mixed) {
        sets = *mixed;
    } else {
        sets.w_s = float(1.0 / s);
        sets.centre_s = mean;
    }
    return dispatch(d, [&](auto t, auto vt) {
        using T = decltype(t);
        constexpr int V = decltype(vt)::value;
        return dispatch_unroll_nt(tuned(g_tuning.dx_unroll, d.dtype == BNS_F32 ? 1 : 2), tuned_nt(g_tuning.dx_nt, 3), [&](auto ut, auto nt) {
            constexpr int U = decltype(ut)::value;
            constexpr int NT = decltype(nt)::value;
            const uint32_t hwv = uint32_t(d.HW / V);
            const uint32_t run_vectors = uint32_t(cg) * hwv;
            const dim3 grid(ceil_div(run_vectors, kBlock * U), uint32_t(d.N));
            BNS_LAUNCH((dx_kernel<T, V, U, NT>), grid, dim3(kBlock), 0, st, static_cast<const T*>(x),
                       static_cast<const T*>(dy), static_cast<T*>(dx), gamma, mean, invstd, dgamma, dbeta,
                       ip, d.C, d.W, d.HW, make_fastdiv(hwv), make_fastdiv(uint32_t(d.W)), c0, run_vectors,
                       sets);
            return hipGetLastError();
        });
    });
}

hipError_t launch_index_boxes(const IndexParams& ip, int C, bns_box* boxes, hipStream_t st) {
    BNS_LAUNCH(index_boxes_kernel, dim3(ceil_div(uint32_t(C), kBlock)), dim3(kBlock), 0, st, ip, C, boxes);
    return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t blocks = (n16 + kBlock * 4 - 1) / (kBlock * 4);
    BNS_LAUNCH(copy_kernel, dim3(uint32_t(blocks)), dim3(kBlock), 0, st, static_cast<const uint4*>(src),
               static_cast<uint4*>(dst), n16);
    return hipGetLastError();
}

}  // namespace bns
