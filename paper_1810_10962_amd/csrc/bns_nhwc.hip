// Kernels for the N x H x W x C layout (the layout the paper writes its tensors in,
// Appendix A: B_l in R^{N x H x W x C}, statistics over dimensions 0, 1, 2).
//
// The tensor is a matrix of M = N*H*W rows and C columns, channels fastest.  Per-channel
// reductions are column sums; the location set S is a set of ROWS: a contiguous block of rows for
// Batch Sampling / NS / VDN, h_cnt runs of w_cnt consecutive rows per sample for Feature Sampling
// (one patch location per layer, as in Alg. 2).  A 128-bit access holds V consecutive channels of
// one row.
//
// All four streaming kernels share one decomposition.  A block is TX column lanes x TY row lanes
// (TX * TY = 256, TX = up to 64 accesses = one wave per row).  Block (tile, k) owns TX * V channels
// and the k-th share of the rows; a thread keeps the per-channel constants of its V channels in
// registers and walks its rows, so the element-wise passes load no parameter twice and divide
// nothing, and the reductions end with one LDS step over the TY row lanes and one partial per
// channel and block: partial[k][c].  The finalize kernels add the partials of a channel in a fixed
// order in fp64, so results are bit-identical from run to run.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "bns_device.hpp"
#include "bns_internal.hpp"

namespace bns {

namespace {

struct Tiling {
    int32_t C, CV;              // channels, channel vectors per row
    int32_t log2_tx, splits;    // TX = 1 << log2_tx column lanes; blocks along the rows
    uint32_t rows_per_block;
};

struct RowSet {                 // the rows of S: sampled row i -> (n, ph, pw) -> row
    int32_t n0, h0, w0;
    int32_t H, W;
    FastDiv patch_div;          // h_cnt * w_cnt
    FastDiv pw_div;             // w_cnt
    uint32_t rows;              // n_cnt * h_cnt * w_cnt
    uint32_t pivot_rows;        // min(kPivotRows, rows)
    float inv_pivot_rows;
    bool contiguous;            // sampled row i = sampled row 0 + i
};

// The one-pass variance is taken about a pivot p_c close to the mean: sum (x - p)^2 / s - (sum (x - p) / s)^2
// loses (1 + 2 k^2) digits' worth for a pivot k standard deviations off.  p_c = mean of the first few
// sampled rows (added in row order, the same expression in the partial and the finalize kernel).
constexpr int kPivotRows = 8;

// The pivot keeps only its upper 16 bits (a bf16 pattern): x - p is then exact for bf16 data and
// carries no low bits that every addition would round the same way.
__device__ __forceinline__ float coarse(float p) { return __uint_as_float(__float_as_uint(p) & 0xFFFF0000u); }

// Accumulation.  A thread adds up to a thousand rows.  Adding them one by one into an fp32 sum loses
// n * eps / 4 of the result when the addends share their low bits (constant dy, activations on a grid,
// exact zeros after a ReLU): every addition then rounds the same way and the errors add up instead of
// averaging out.  So the rows of one unrolled iteration are added in fp32 and each group's sum goes
// into an fp64 accumulator (one fp64 add per group and channel: far below the fp64 rate).

__device__ __forceinline__ uint32_t sampled_row(const RowSet& s, uint32_t i) {
    const uint32_t n = fdiv(i, s.patch_div);
    const uint32_t r = i - n * s.patch_div.d;
    const uint32_t ph = fdiv(r, s.pw_div);
    const uint32_t pw = r - ph * s.pw_div.d;
    return ((uint32_t(s.n0) + n) * uint32_t(s.H) + uint32_t(s.h0) + ph) * uint32_t(s.W) + uint32_t(s.w0) + pw;
}

struct Lane {
    int tx, ty, TY, k, cv;
    bool live;
};

__device__ __forceinline__ Lane lane_of(const Tiling& t) {
    Lane l;
    const int TX = 1 << t.log2_tx;
    l.TY = kBlock >> t.log2_tx;
    l.tx = threadIdx.x & (TX - 1);
    l.ty = threadIdx.x >> t.log2_tx;
    const int tile = blockIdx.x / t.splits;
    l.k = blockIdx.x - tile * t.splits;
    l.cv = tile * TX + l.tx;
    l.live = l.cv < t.CV;
    return l;
}

// Adds a[], q[] over the TY row lanes of the block (fixed order) and writes one partial per channel.
template <int V>
__device__ __forceinline__ void write_partials(float (&a)[V], float (&q)[V], float* lds, const Tiling& t, const Lane& l,
                                               Partial* __restrict__ partial) {
    const int stride = (1 << t.log2_tx) * V;            // floats per row lane; lds: [2][TY][stride]
#pragma unroll
    for (int i = 0; i < V; ++i) {
        lds[l.ty * stride + l.tx * V + i] = a[i];
        lds[(l.TY + l.ty) * stride + l.tx * V + i] = q[i];
    }
    __syncthreads();
    if (l.ty != 0 || !l.live) return;
#pragma unroll
    for (int i = 0; i < V; ++i) {
        float sa = lds[l.tx * V + i], sq = lds[l.TY * stride + l.tx * V + i];
        for (int r = 1; r < l.TY; ++r) {
            sa += lds[r * stride + l.tx * V + i];
            sq += lds[(l.TY + r) * stride + l.tx * V + i];
        }
        partial[size_t(l.k) * t.C + size_t(l.cv) * V + i] = Partial{sa, sq};
    }
}

// Forward statistics (Eq. 3): partial[k][c] = (sum (x - p_c), sum (x - p_c)^2) over the k-th share of
// S, p_c = mean of x over the first few sampled rows.
//
// A row lane takes its rows kStatRows at a time.  The loads of the next batch are issued before the
// current one is added up, and the pivot rows travel together with the first batch, so a block with few
// rows (a small S spread over the whole device) waits for memory once and a block with many rows keeps
// two batches in flight.  Row indices past the end of the share are clamped to its last row and their
// terms dropped, so every load is unconditional.  CONTIG: the rows of S are one contiguous run (Batch
// Sampling, full BN, NS, the virtual set), so the sampled row needs no division.  KEEP: loads without the
// non-temporal hint, so that the normalization pass finds the rows of S in the memory-side cache.
constexpr int kStatRows = 8;

template <typename T, int V, bool CONTIG, bool KEEP>
__global__ __launch_bounds__(kBlock) void nhwc_stats_partial_kernel(const T* __restrict__ x,
                                                                    Partial* __restrict__ partial, RowSet S, Tiling t) {
    __shared__ float lds[2 * kBlock * V];
    __shared__ float piv[kWave * V];                             // at most 64 column lanes
    const Lane l = lane_of(t);
    const uint32_t i0 = uint32_t(l.k) * t.rows_per_block;
    const uint32_t i1 = min(i0 + t.rows_per_block, S.rows);      // i1 > i0: no block is empty
    const uint32_t TY = uint32_t(l.TY);
    const uint32_t step = uint32_t(kStatRows) * TY;
    const uint32_t batches = (i1 - i0 + step - 1u) / step;      // the same for every thread of the block
    float a[V], q[V], p[V];
    double A[V], Q[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        a[e] = q[e] = p[e] = 0.f;
        A[e] = Q[e] = 0.0;
    }
    {
        // (lanes past the last channel vector repeat it: they take part in the barrier below and write nothing)
        const T* xc = x + size_t(l.live ? l.cv : t.CV - 1) * V;
        const uint32_t first = sampled_row(S, 0u);
        auto row_of = [&](uint32_t i) { return CONTIG ? first + i : sampled_row(S, i); };
        auto fetch = [&](Vec<T, V>(&v)[kStatRows], uint32_t i) {
#pragma unroll
            for (int u = 0; u < kStatRows; ++u) {
                const T* p = xc + size_t(row_of(min(i + uint32_t(u) * TY, i1 - 1u))) * t.C;
                if (KEEP) v[u].load(p); else v[u].load_nt(p);
            }
        };
        auto add = [&](const Vec<T, V>(&v)[kStatRows], uint32_t i) {
            if (i + uint32_t(kStatRows - 1) * TY < i1) {         // every row of the batch belongs to the share
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    float d[kStatRows];
#pragma unroll
                    for (int u = 0; u < kStatRows; ++u) d[u] = v[u].f[e] - p[e];
                    A[e] += double(((d[0] + d[1]) + (d[2] + d[3])) + ((d[4] + d[5]) + (d[6] + d[7])));
                    float sq = d[0] * d[0];
#pragma unroll
                    for (int u = 1; u < kStatRows; ++u) sq = fmaf(d[u], d[u], sq);
                    Q[e] += double(sq);
                }
            } else {
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    float d[kStatRows];
#pragma unroll
                    for (int u = 0; u < kStatRows; ++u) d[u] = i + uint32_t(u) * TY < i1 ? v[u].f[e] - p[e] : 0.f;
                    A[e] += double(((d[0] + d[1]) + (d[2] + d[3])) + ((d[4] + d[5]) + (d[6] + d[7])));
                    float sq = d[0] * d[0];
#pragma unroll
                    for (int u = 1; u < kStatRows; ++u) sq = fmaf(d[u], d[u], sq);
                    Q[e] += double(sq);
                }
            }
        };
        static_assert(kStatRows == 8, "the sums above are written out for eight rows");
        Vec<T, V> pv[kPivotRows], v0[kStatRows], v1[kStatRows];
        uint32_t i = i0 + uint32_t(l.ty);
        // The pivot rows are the same few rows for every block of the launch: only the first row lane of a block
        // reads them and hands the pivots to the others through LDS (every thread of every block reading them put
        // thousands of requests on the few L2 channels that hold those rows).
        if (l.ty == 0) {
#pragma unroll
            for (int j = 0; j < kPivotRows; ++j)     // no branches: all loads in flight together
                pv[j].load(xc + size_t(row_of(min(uint32_t(j), S.pivot_rows - 1u))) * t.C);
        }
        fetch(v0, i);
        if (l.ty == 0) {
#pragma unroll
            for (int j = 0; j < kPivotRows; ++j)
#pragma unroll
                for (int e = 0; e < V; ++e) p[e] += uint32_t(j) < S.pivot_rows ? pv[j].f[e] : 0.f;
#pragma unroll
            for (int e = 0; e < V; ++e) piv[l.tx * V + e] = coarse(p[e] * S.inv_pivot_rows);
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < V; ++e) p[e] = piv[l.tx * V + e];
        for (uint32_t b = 0; b < batches; b += 2u) {
            if (b + 1u < batches) fetch(v1, i + step);
            add(v0, i);
            if (b + 1u < batches) {
                if (b + 2u < batches) fetch(v0, i + 2u * step);
                add(v1, i + step);
            }
            i += 2u * step;
        }
#pragma unroll
        for (int e = 0; e < V; ++e) {
            a[e] = float(A[e]);
            q[e] = float(Q[e]);
        }
    }
    write_partials<V>(a, q, lds, t, l, partial);
}

struct RowBox {                 // membership of a row in S
    uint32_t n0, n1, h0, h1, w0, w1;
    FastDiv hw_div, w_div;
};

__device__ __forceinline__ bool row_in(const RowBox& b, uint32_t row) {
    const uint32_t n = fdiv(row, b.hw_div);
    const uint32_t rem = row - n * b.hw_div.d;
    const uint32_t h = fdiv(rem, b.w_div);
    const uint32_t w = rem - h * b.w_div.d;
    return n >= b.n0 && n < b.n1 && h >= b.h0 && h < b.h1 && w >= b.w0 && w < b.w1;
}

// Backward sums of Eq. 5 over all M rows: partial[k][c] = (sum dy, sum dy * (x - mean_c)).
// OUTSIDE: the kernel also writes dx on the rows that are NOT in S.  The second branch of Eq. 6, dx = gamma r dy,
// needs none of the sums, and dy of those rows is in registers here anyway; what is left for after the sums are
// the rows of S alone (nhwc_dx_rows_kernel).  Backward then has to move (3 + 2r) e bytes per element instead of (4 + r) e.
// KEEP: what the dx pass reads again is loaded without the non-temporal hint, so that it stays in the memory-side
// cache: 1 = dy in the blocks of the first `keep_splits` row shares (as many as fit; the dx pass loads and stores
// with the hint, so what is cached stays until it gets there), 2 = dy and x everywhere (S is most of the rows and
// both fit), 0 = neither (dx is written here).
template <typename T, int V, bool OUTSIDE, int KEEP>
__device__ __forceinline__ void reduce_partial_body(const T* __restrict__ x, const T* __restrict__ dy,
                                                    const float* __restrict__ mean, Partial* __restrict__ partial,
                                                    const Tiling& t, uint32_t M, T* __restrict__ dx,
                                                    const float* __restrict__ gamma, const float* __restrict__ invstd,
                                                    const RowBox& B, float* lds, uint32_t keep_splits) {
    const Lane l = lane_of(t);
    const uint32_t r0 = uint32_t(l.k) * t.rows_per_block;
    const uint32_t r1 = min(r0 + t.rows_per_block, M);
    const uint32_t TY = uint32_t(l.TY);
    float a[V], q[V], mu[V], sc[V];
    double A[V], Q[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        a[e] = q[e] = mu[e] = sc[e] = 0.f;
        A[e] = Q[e] = 0.0;
    }
    if (l.live) {
#pragma unroll
        for (int e = 0; e < V; ++e) mu[e] = mean[l.cv * V + e];
        if (OUTSIDE) {
#pragma unroll
            for (int e = 0; e < V; ++e) sc[e] = gamma[l.cv * V + e] * invstd[l.cv * V + e];      // a = gamma r
        }
        const size_t col = size_t(l.cv) * V;
        auto walk = [&](auto keep_dy, auto keep_x) {
            constexpr bool KD = decltype(keep_dy)::value, KX = decltype(keep_x)::value;
            uint32_t r = r0 + uint32_t(l.ty);
            for (; r + TY < r1; r += 2u * TY) {
                Vec<T, V> g[2], v[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const size_t off = size_t(r + uint32_t(u) * TY) * t.C + col;
                    if (KD) g[u].load(dy + off); else g[u].load_nt(dy + off);
                    if (KX) v[u].load(x + off); else v[u].load_nt(x + off);
                }
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    A[e] += double(g[0].f[e] + g[1].f[e]);
                    Q[e] += double(fmaf(g[1].f[e], v[1].f[e] - mu[e], g[0].f[e] * (v[0].f[e] - mu[e])));
                }
                if (OUTSIDE) {
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const uint32_t row = r + uint32_t(u) * TY;
                        if (!row_in(B, row)) {
#pragma unroll
                            for (int e = 0; e < V; ++e) g[u].f[e] *= sc[e];
                            g[u].store_nt(dx + size_t(row) * t.C + col);
                        }
                    }
                }
            }
            for (; r < r1; r += TY) {
                const size_t off = size_t(r) * t.C + col;
                Vec<T, V> g, v;
                if (KD) g.load(dy + off); else g.load_nt(dy + off);
                if (KX) v.load(x + off); else v.load_nt(x + off);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    A[e] += double(g.f[e]);
                    Q[e] += double(g.f[e] * (v.f[e] - mu[e]));
                }
                if (OUTSIDE && !row_in(B, r)) {
#pragma unroll
                    for (int e = 0; e < V; ++e) g.f[e] *= sc[e];
                    g.store_nt(dx + off);
                }
            }
        };
        if constexpr (KEEP == 2) {
            walk(std::true_type(), std::true_type());
        } else if constexpr (KEEP == 1) {
            if (uint32_t(l.k) < keep_splits) walk(std::true_type(), std::false_type());      // (the same for the whole block)
            else walk(std::false_type(), std::false_type());
        } else {
            walk(std::false_type(), std::false_type());
        }
#pragma unroll
        for (int e = 0; e < V; ++e) {
            a[e] = float(A[e]);
            q[e] = float(Q[e]);
        }
    }
    write_partials<V>(a, q, lds, t, l, partial);
}

template <typename T, int V, int KEEP>
__global__ __launch_bounds__(kBlock) void nhwc_reduce_partial_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                                     const float* __restrict__ mean,
                                                                     Partial* __restrict__ partial, Tiling t, uint32_t M,
                                                                     uint32_t keep_splits) {
    __shared__ float lds[2 * kBlock * V];
    reduce_partial_body<T, V, false, KEEP>(x, dy, mean, partial, t, M, nullptr, nullptr, nullptr, RowBox{}, lds, keep_splits);
}

template <typename T, int V>
__global__ __launch_bounds__(kBlock) void nhwc_reduce_outside_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                                     const float* __restrict__ mean,
                                                                     Partial* __restrict__ partial, Tiling t, uint32_t M,
                                                                     T* __restrict__ dx, const float* __restrict__ gamma,
                                                                     const float* __restrict__ invstd, RowBox B) {
    __shared__ float lds[2 * kBlock * V];
    reduce_partial_body<T, V, true, 0>(x, dy, mean, partial, t, M, dx, gamma, invstd, B, lds, 0u);
}

// Finalize kernels: a block takes kFinCh neighbouring channels; thread (ch, kl) adds the partials
// k = kl, kl + kFinK, ... of channel ch in fp64 (a wave reads whole 64-byte runs of partial[k][.]),
// then thread ch adds the kFinK lane sums in index order.
constexpr int kFinCh = 8;
constexpr int kFinK = kBlock / kFinCh;

// The thread that sum_splits returns true for, and its channel.
__device__ __forceinline__ int led_channel() { return blockIdx.x * kFinCh + int(threadIdx.x % kFinCh); }
__device__ __forceinline__ bool leads_channel(int C) { return threadIdx.x / kFinCh == 0 && led_channel() < C; }

__device__ __forceinline__ bool sum_splits(const Partial* __restrict__ partial, int C, int splits, double* lds, int& c,
                                           double& s1, double& s2) {
    const int ch = threadIdx.x % kFinCh, kl = threadIdx.x / kFinCh;
    c = blockIdx.x * kFinCh + ch;
    double a = 0.0, b = 0.0;
    if (c < C) {
        int k = kl;
        for (; k + 15 * kFinK < splits; k += 16 * kFinK) {     // sixteen loads in flight, added in index order
            Partial p[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) p[u] = partial[size_t(k + u * kFinK) * C + c];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                a += double(p[u].a);
                b += double(p[u].b);
            }
        }
        for (; k < splits; k += kFinK) {
            const Partial p = partial[size_t(k) * C + c];
            a += double(p.a);
            b += double(p.b);
        }
    }
    lds[kl * kFinCh + ch] = a;
    lds[(kFinK + kl) * kFinCh + ch] = b;
    __syncthreads();
    if (kl != 0 || c >= C) return false;
    s1 = lds[ch];
    s2 = lds[kFinK * kFinCh + ch];
    for (int j = 1; j < kFinK; ++j) {
        s1 += lds[j * kFinCh + ch];
        s2 += lds[(kFinK + j) * kFinCh + ch];
    }
    return true;
}

// The pivot of channel c, the same expression as in nhwc_stats_partial_kernel.
template <typename T>
__device__ __forceinline__ float column_pivot(const T* __restrict__ x, const RowSet& S, int C, int c) {
    float pv[kPivotRows], psum = 0.f;
#pragma unroll
    for (int j = 0; j < kPivotRows; ++j)
        pv[j] = load_scalar<T>(x + size_t(sampled_row(S, min(uint32_t(j), S.pivot_rows - 1u))) * C + c);
#pragma unroll
    for (int j = 0; j < kPivotRows; ++j) psum += uint32_t(j) < S.pivot_rows ? pv[j] : 0.f;
    return coarse(psum * S.inv_pivot_rows);
}

template <typename T>
__global__ __launch_bounds__(kBlock) void nhwc_stats_finalize_kernel(
    const T* __restrict__ x, const Partial* __restrict__ partial, RowSet S, int C, int splits, float eps, float momentum,
    float* __restrict__ save_mean, float* __restrict__ save_invstd, float* __restrict__ running_mean,
    float* __restrict__ running_var) {
    __shared__ double lds[2 * kBlock];
    int c;
    double s1, s2;
    const float pivot_f = leads_channel(C) ? column_pivot(x, S, C, led_channel()) : 0.f;   // loads overlap the sums'
    if (!sum_splits(partial, C, splits, lds, c, s1, s2)) return;
    const double pivot = double(pivot_f);
    const double s = double(S.rows);
    const double m1 = s1 / s;
    const double mean = pivot + m1;
    double var = s2 / s - m1 * m1;      // biased (1/s), Eq. 3
    if (var < 0.0) var = 0.0;
    save_mean[c] = float(mean);
    save_invstd[c] = float(1.0 / sqrt(var + double(eps)));
    const double al = double(momentum);                       // Eq. 8
    if (running_mean) running_mean[c] = float((1.0 - al) * double(running_mean[c]) + al * mean);
    if (running_var) running_var[c] = float((1.0 - al) * double(running_var[c]) + al * var);
}

// "VDN + sampling" (Eq. 4): the sums of the sampled real set S and of the virtual set V (the first n_v
// samples), each into its own E and Var by Eq. 3, then the blend.  Two passes of sum_splits over the same
// LDS, every thread taking part in both.
template <typename T>
__global__ __launch_bounds__(kBlock) void nhwc_stats_finalize_mixed_kernel(
    const T* __restrict__ x, const Partial* __restrict__ partial_s, int splits_s, const Partial* __restrict__ partial_v,
    int splits_v, RowSet S, RowSet Vs, int C, float mix_beta, float eps, float momentum, float* __restrict__ save_mean,
    float* __restrict__ save_invstd, float* __restrict__ mean_parts, float* __restrict__ running_mean,
    float* __restrict__ running_var) {
    __shared__ double lds[2 * kBlock];
    int c;
    double a1 = 0.0, a2 = 0.0, v1 = 0.0, v2 = 0.0;
    const bool lead = leads_channel(C);
    const float pivot_s = lead ? column_pivot(x, S, C, led_channel()) : 0.f;
    const float pivot_v = lead ? column_pivot(x, Vs, C, led_channel()) : 0.f;
    const bool lead_s = sum_splits(partial_s, C, splits_s, lds, c, a1, a2);
    __syncthreads();                                            // the leaders have read their sums
    const bool lead_v = sum_splits(partial_v, C, splits_v, lds, c, v1, v2);
    if (!lead_s || !lead_v) return;
    const double ss = double(S.rows), sv = double(Vs.rows);
    const double ms = a1 / ss, mv = v1 / sv;
    const double e_s = double(pivot_s) + ms;
    const double e_v = double(pivot_v) + mv;
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
    const double al = double(momentum);                         // Eq. 8
    if (running_mean) running_mean[c] = float((1.0 - al) * double(running_mean[c]) + al * mean);
    if (running_var) running_var[c] = float((1.0 - al) * double(running_var[c]) + al * var);
}

__global__ __launch_bounds__(kBlock) void nhwc_reduce_finalize_kernel(const Partial* __restrict__ partial, int C,
                                                                      int splits, const float* __restrict__ invstd,
                                                                      float* __restrict__ dgamma,
                                                                      float* __restrict__ dbeta) {
    __shared__ double lds[2 * kBlock];
    int c;
    double s1, s2;
    const float r = leads_channel(C) ? invstd[led_channel()] : 0.f;
    if (!sum_splits(partial, C, splits, lds, c, s1, s2)) return;
    dbeta[c] = float(s1);
    dgamma[c] = float(s2 * double(r));
}

// Eq. 1 on every element.  var_eps >= 0: `invstd` holds variances (inference, Appendix D).
template <typename T, int V>
__global__ __launch_bounds__(kBlock) void nhwc_normalize_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                                const float* __restrict__ gamma,
                                                                const float* __restrict__ beta,
                                                                const float* __restrict__ mean,
                                                                const float* __restrict__ invstd, Tiling t, uint32_t M,
                                                                float var_eps) {
    const Lane l = lane_of(t);
    if (!l.live) return;
    const uint32_t r0 = uint32_t(l.k) * t.rows_per_block;
    const uint32_t r1 = min(r0 + t.rows_per_block, M);
    const uint32_t TY = uint32_t(l.TY);
    float sc[V], mu[V], be[V], rs[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {       // every load first: one round trip to memory, not one per channel
        const int c = l.cv * V + e;
        sc[e] = gamma[c];
        rs[e] = invstd[c];
        mu[e] = mean[c];
        be[e] = beta[c];
    }
    if (var_eps >= 0.f) {
#pragma unroll
        for (int e = 0; e < V; ++e) rs[e] = 1.0f / sqrtf(rs[e] + var_eps);
    }
#pragma unroll
    for (int e = 0; e < V; ++e) sc[e] *= rs[e];
    const size_t col = size_t(l.cv) * V;
    uint32_t r = r0 + uint32_t(l.ty);
    for (; r + 3u * TY < r1; r += 4u * TY) {
        Vec<T, V> v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u].load_nt(x + size_t(r + uint32_t(u) * TY) * t.C + col);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int e = 0; e < V; ++e) v[u].f[e] = fmaf(v[u].f[e] - mu[e], sc[e], be[e]);
            v[u].store_nt(y + size_t(r + uint32_t(u) * TY) * t.C + col);
        }
    }
    for (; r < r1; r += TY) {
        Vec<T, V> v;
        v.load_nt(x + size_t(r) * t.C + col);
#pragma unroll
        for (int e = 0; e < V; ++e) v.f[e] = fmaf(v.f[e] - mu[e], sc[e], be[e]);
        v.store_nt(y + size_t(r) * t.C + col);
    }
}

// Eq. 6 on every element: rows outside S scale dy, rows in S also read x and take the 1/s terms.
//   dx = a g                                   a  = gamma r
//   dx = a g - (k1 (x - mean) + k2)            k1 = a r dgamma / s,  k2 = a dbeta / s
template <typename T, int V>
__global__ __launch_bounds__(kBlock) void nhwc_dx_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                         T* __restrict__ dx, const float* __restrict__ gamma,
                                                         const float* __restrict__ mean,
                                                         const float* __restrict__ invstd,
                                                         const float* __restrict__ dgamma,
                                                         const float* __restrict__ dbeta, RowBox B, Tiling t,
                                                         uint32_t M, float inv_s) {
    const Lane l = lane_of(t);
    if (!l.live) return;
    const uint32_t r0 = uint32_t(l.k) * t.rows_per_block;
    const uint32_t r1 = min(r0 + t.rows_per_block, M);
    const uint32_t TY = uint32_t(l.TY);
    float a[V], mu[V], k1[V], k2[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        const int c = l.cv * V + e;
        const float r = invstd[c];
        a[e] = gamma[c] * r;
        mu[e] = mean[c];
        k1[e] = a[e] * inv_s * (dgamma[c] * r);
        k2[e] = a[e] * inv_s * dbeta[c];
    }
    const size_t col = size_t(l.cv) * V;
    uint32_t r = r0 + uint32_t(l.ty);
    for (; r + 3u * TY < r1; r += 4u * TY) {
        Vec<T, V> g[4], v[4];
        bool in[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t row = r + uint32_t(u) * TY;
            g[u].load_nt(dy + size_t(row) * t.C + col);
            in[u] = row_in(B, row);
            if (in[u]) v[u].load_nt(x + size_t(row) * t.C + col);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (in[u]) {
#pragma unroll
                for (int e = 0; e < V; ++e) g[u].f[e] = fmaf(a[e], g[u].f[e], -fmaf(k1[e], v[u].f[e] - mu[e], k2[e]));
            } else {
#pragma unroll
                for (int e = 0; e < V; ++e) g[u].f[e] *= a[e];
            }
            g[u].store_nt(dx + size_t(r + uint32_t(u) * TY) * t.C + col);
        }
    }
    for (; r < r1; r += TY) {
        Vec<T, V> g;
        g.load_nt(dy + size_t(r) * t.C + col);
        if (row_in(B, r)) {
            Vec<T, V> v;
            v.load_nt(x + size_t(r) * t.C + col);
#pragma unroll
            for (int e = 0; e < V; ++e) g.f[e] = fmaf(a[e], g.f[e], -fmaf(k1[e], v.f[e] - mu[e], k2[e]));
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) g.f[e] *= a[e];
        }
        g.store_nt(dx + size_t(r) * t.C + col);
    }
}

// Eq. 6, first branch, on the rows of S alone (sampled row i of the k-th share, as in the statistics kernel); the
// other rows were written by nhwc_reduce_outside_kernel.
template <typename T, int V, bool CONTIG>
__global__ __launch_bounds__(kBlock) void nhwc_dx_rows_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                              T* __restrict__ dx, const float* __restrict__ gamma,
                                                              const float* __restrict__ mean,
                                                              const float* __restrict__ invstd,
                                                              const float* __restrict__ dgamma,
                                                              const float* __restrict__ dbeta, RowSet S, Tiling t,
                                                              float inv_s) {
    const Lane l = lane_of(t);
    if (!l.live) return;
    const uint32_t i0 = uint32_t(l.k) * t.rows_per_block;
    const uint32_t i1 = min(i0 + t.rows_per_block, S.rows);
    const uint32_t TY = uint32_t(l.TY);
    float a[V], mu[V], k1[V], k2[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        const int c = l.cv * V + e;
        const float r = invstd[c];
        a[e] = gamma[c] * r;
        mu[e] = mean[c];
        k1[e] = a[e] * inv_s * (dgamma[c] * r);
        k2[e] = a[e] * inv_s * dbeta[c];
    }
    const size_t col = size_t(l.cv) * V;
    const uint32_t first = sampled_row(S, 0u);
    auto row_of = [&](uint32_t i) { return CONTIG ? first + i : sampled_row(S, i); };
    uint32_t i = i0 + uint32_t(l.ty);
    for (; i + 3u * TY < i1; i += 4u * TY) {
        Vec<T, V> g[4], v[4];
        size_t off[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            off[u] = size_t(row_of(i + uint32_t(u) * TY)) * t.C + col;
            g[u].load_nt(dy + off[u]);
            v[u].load_nt(x + off[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int e = 0; e < V; ++e) g[u].f[e] = fmaf(a[e], g[u].f[e], -fmaf(k1[e], v[u].f[e] - mu[e], k2[e]));
            g[u].store_nt(dx + off[u]);
        }
    }
    for (; i < i1; i += TY) {
        const size_t off = size_t(row_of(i)) * t.C + col;
        Vec<T, V> g, v;
        g.load_nt(dy + off);
        v.load_nt(x + off);
#pragma unroll
        for (int e = 0; e < V; ++e) g.f[e] = fmaf(a[e], g.f[e], -fmaf(k1[e], v.f[e] - mu[e], k2[e]));
        g.store_nt(dx + off);
    }
}

// Backward of Eq. 4: rows of the first n_v samples belong to the virtual set (weight w_v = mix_beta / s_v,
// centre E[x_v]), rows of S to the sampled real set (w_s = (1 - mix_beta) / s_s, centre E[x_s]):
//   dx = a g - a w (dbeta + r dgamma (x - E_set)),   dx = a g elsewhere.
template <typename T, int V>
__global__ __launch_bounds__(kBlock) void nhwc_dx_mixed_kernel(
    const T* __restrict__ x, const T* __restrict__ dy, T* __restrict__ dx, const float* __restrict__ gamma,
    const float* __restrict__ invstd, const float* __restrict__ dgamma, const float* __restrict__ dbeta,
    const float* __restrict__ centre_v, const float* __restrict__ centre_s, RowBox B, uint32_t virtual_rows, float w_v,
    float w_s, Tiling t, uint32_t M) {
    const Lane l = lane_of(t);
    if (!l.live) return;
    const uint32_t r0 = uint32_t(l.k) * t.rows_per_block;
    const uint32_t r1 = min(r0 + t.rows_per_block, M);
    const uint32_t TY = uint32_t(l.TY);
    float a[V], cv_[V], cs_[V], k1[V], k2[V];          // k1, k2 per unit weight
#pragma unroll
    for (int e = 0; e < V; ++e) {
        const int c = l.cv * V + e;
        const float r = invstd[c];
        a[e] = gamma[c] * r;
        cv_[e] = centre_v[c];
        cs_[e] = centre_s[c];
        k1[e] = a[e] * (dgamma[c] * r);
        k2[e] = a[e] * dbeta[c];
    }
    const size_t col = size_t(l.cv) * V;
    for (uint32_t r = r0 + uint32_t(l.ty); r < r1; r += TY) {
        Vec<T, V> g;
        g.load_nt(dy + size_t(r) * t.C + col);
        const bool virt = r < virtual_rows;
        if (virt || row_in(B, r)) {
            Vec<T, V> v;
            v.load_nt(x + size_t(r) * t.C + col);
            const float w = virt ? w_v : w_s;
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float centre = virt ? cv_[e] : cs_[e];
                g.f[e] = fmaf(a[e], g.f[e], -w * fmaf(k1[e], v.f[e] - centre, k2[e]));
            }
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) g.f[e] *= a[e];
        }
        g.store_nt(dx + size_t(r) * t.C + col);
    }
}

// ---- small tensors: one launch per direction ---------------------------------------------------
// A block owns TX * V channels and ALL rows, so nothing crosses blocks: pass 1 adds the block's columns
// (the rows of S forward, all rows backward), one LDS step over the row lanes gives every thread the
// totals of its columns, pass 2 walks all rows again (the tensor is small: that read comes from cache).
// At most kNhwcSmallRows rows per row lane, so the fp32 sums are short.

// On return a[], q[] hold the block totals of the thread's columns, the same bits in every row lane.
template <int V>
__device__ __forceinline__ void block_column_sums(float (&a)[V], float (&q)[V], float* lds, const Tiling& t,
                                                  const Lane& l) {
    const int stride = (1 << t.log2_tx) * V;
#pragma unroll
    for (int i = 0; i < V; ++i) {
        lds[l.ty * stride + l.tx * V + i] = a[i];
        lds[(l.TY + l.ty) * stride + l.tx * V + i] = q[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < V; ++i) {
        float sa = lds[l.tx * V + i], sq = lds[l.TY * stride + l.tx * V + i];
        for (int r = 1; r < l.TY; ++r) {
            sa += lds[r * stride + l.tx * V + i];
            sq += lds[(l.TY + r) * stride + l.tx * V + i];
        }
        a[i] = sa;
        q[i] = sq;
    }
}

// Eq. 3, Eq. 8 and Eq. 1 in one launch.
template <typename T, int V>
__global__ __launch_bounds__(kBlock) void nhwc_small_forward_kernel(
    const T* __restrict__ x, T* __restrict__ y, const float* __restrict__ gamma, const float* __restrict__ beta, RowSet S,
    Tiling t, uint32_t M, float eps, float momentum, float* __restrict__ save_mean, float* __restrict__ save_invstd,
    float* __restrict__ running_mean, float* __restrict__ running_var) {
    __shared__ float lds[2 * kBlock * V];
    const Lane l = lane_of(t);
    const uint32_t TY = uint32_t(l.TY);
    const size_t col = size_t(l.live ? l.cv : 0) * V;
    float a[V], q[V], p[V];
#pragma unroll
    for (int e = 0; e < V; ++e) a[e] = q[e] = p[e] = 0.f;
    if (l.live) {
        Vec<T, V> pv[kPivotRows];
#pragma unroll
        for (int j = 0; j < kPivotRows; ++j)
            pv[j].load(x + size_t(sampled_row(S, min(uint32_t(j), S.pivot_rows - 1u))) * t.C + col);
#pragma unroll
        for (int j = 0; j < kPivotRows; ++j)
#pragma unroll
            for (int e = 0; e < V; ++e) p[e] += uint32_t(j) < S.pivot_rows ? pv[j].f[e] : 0.f;
#pragma unroll
        for (int e = 0; e < V; ++e) p[e] = coarse(p[e] * S.inv_pivot_rows);
        uint32_t i = uint32_t(l.ty);
        for (; i + 3u * TY < S.rows; i += 4u * TY) {
            Vec<T, V> v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u].load(x + size_t(sampled_row(S, i + uint32_t(u) * TY)) * t.C + col);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const float dlt = v[u].f[e] - p[e];
                    a[e] += dlt;
                    q[e] = fmaf(dlt, dlt, q[e]);
                }
        }
        for (; i < S.rows; i += TY) {
            Vec<T, V> v;
            v.load(x + size_t(sampled_row(S, i)) * t.C + col);
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float dlt = v.f[e] - p[e];
                a[e] += dlt;
                q[e] = fmaf(dlt, dlt, q[e]);
            }
        }
    }
    block_column_sums<V>(a, q, lds, t, l);
    if (!l.live) return;
    float mu[V], sc[V], be[V];
    const double s = double(S.rows), al = double(momentum);
#pragma unroll
    for (int e = 0; e < V; ++e) {
        const int c = l.cv * V + e;
        const double m1 = double(a[e]) / s;
        const double mean = double(p[e]) + m1;
        double var = double(q[e]) / s - m1 * m1;      // biased (1/s), Eq. 3
        if (var < 0.0) var = 0.0;
        mu[e] = float(mean);
        const float r = float(1.0 / sqrt(var + double(eps)));
        sc[e] = gamma[c] * r;
        be[e] = beta[c];
        if (l.ty == 0) {
            save_mean[c] = mu[e];
            save_invstd[c] = r;
            if (running_mean) running_mean[c] = float((1.0 - al) * double(running_mean[c]) + al * mean);     // Eq. 8
            if (running_var) running_var[c] = float((1.0 - al) * double(running_var[c]) + al * var);
        }
    }
    uint32_t r = uint32_t(l.ty);
    for (; r + 3u * TY < M; r += 4u * TY) {
        Vec<T, V> v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u].load(x + size_t(r + uint32_t(u) * TY) * t.C + col);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int e = 0; e < V; ++e) v[u].f[e] = fmaf(v[u].f[e] - mu[e], sc[e], be[e]);
            v[u].store_nt(y + size_t(r + uint32_t(u) * TY) * t.C + col);
        }
    }
    for (; r < M; r += TY) {
        Vec<T, V> v;
        v.load(x + size_t(r) * t.C + col);
#pragma unroll
        for (int e = 0; e < V; ++e) v.f[e] = fmaf(v.f[e] - mu[e], sc[e], be[e]);
        v.store_nt(y + size_t(r) * t.C + col);
    }
}

// The sums of Eq. 5 and Eq. 6 in one launch.
template <typename T, int V>
__global__ __launch_bounds__(kBlock) void nhwc_small_backward_kernel(
    const T* __restrict__ x, const T* __restrict__ dy, T* __restrict__ dx, const float* __restrict__ gamma,
    const float* __restrict__ mean, const float* __restrict__ invstd, float* __restrict__ dgamma,
    float* __restrict__ dbeta, RowBox B, Tiling t, uint32_t M, float inv_s) {
    __shared__ float lds[2 * kBlock * V];
    const Lane l = lane_of(t);
    const uint32_t TY = uint32_t(l.TY);
    const size_t col = size_t(l.live ? l.cv : 0) * V;
    float a[V], q[V], mu[V], rs[V], ga[V];
#pragma unroll
    for (int e = 0; e < V; ++e) a[e] = q[e] = mu[e] = rs[e] = ga[e] = 0.f;
    if (l.live) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
            mu[e] = mean[l.cv * V + e];
            rs[e] = invstd[l.cv * V + e];
            ga[e] = gamma[l.cv * V + e];
        }
        uint32_t r = uint32_t(l.ty);
        for (; r + TY < M; r += 2u * TY) {
            Vec<T, V> g[2], v[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const size_t off = size_t(r + uint32_t(u) * TY) * t.C + col;
                g[u].load(dy + off);
                v[u].load(x + off);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    a[e] += g[u].f[e];
                    q[e] = fmaf(g[u].f[e], v[u].f[e] - mu[e], q[e]);
                }
        }
        for (; r < M; r += TY) {
            const size_t off = size_t(r) * t.C + col;
            Vec<T, V> g, v;
            g.load(dy + off);
            v.load(x + off);
#pragma unroll
            for (int e = 0; e < V; ++e) {
                a[e] += g.f[e];
                q[e] = fmaf(g.f[e], v.f[e] - mu[e], q[e]);
            }
        }
    }
    block_column_sums<V>(a, q, lds, t, l);
    if (!l.live) return;
    float k1[V], k2[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        const int c = l.cv * V + e;
        const float db = a[e];
        const float dg = float(double(q[e]) * double(rs[e]));
        if (l.ty == 0) {
            dbeta[c] = db;
            dgamma[c] = dg;
        }
        ga[e] *= rs[e];                                  // a = gamma r
        k1[e] = ga[e] * inv_s * (dg * rs[e]);
        k2[e] = ga[e] * inv_s * db;
    }
    uint32_t r = uint32_t(l.ty);
    for (; r + TY < M; r += 2u * TY) {
        Vec<T, V> g[2], v[2];
        bool in[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t row = r + uint32_t(u) * TY;
            g[u].load(dy + size_t(row) * t.C + col);
            in[u] = row_in(B, row);
            if (in[u]) v[u].load(x + size_t(row) * t.C + col);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (in[u]) {
#pragma unroll
                for (int e = 0; e < V; ++e) g[u].f[e] = fmaf(ga[e], g[u].f[e], -fmaf(k1[e], v[u].f[e] - mu[e], k2[e]));
            } else {
#pragma unroll
                for (int e = 0; e < V; ++e) g[u].f[e] *= ga[e];
            }
            g[u].store_nt(dx + size_t(r + uint32_t(u) * TY) * t.C + col);
        }
    }
    for (; r < M; r += TY) {
        Vec<T, V> g;
        g.load(dy + size_t(r) * t.C + col);
        if (row_in(B, r)) {
            Vec<T, V> v;
            v.load(x + size_t(r) * t.C + col);
#pragma unroll
            for (int e = 0; e < V; ++e) g.f[e] = fmaf(ga[e], g.f[e], -fmaf(k1[e], v.f[e] - mu[e], k2[e]));
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) g.f[e] *= ga[e];
        }
        g.store_nt(dx + size_t(r) * t.C + col);
    }
}

inline uint32_t ceil_div_u(uint32_t a, uint32_t b) { return uint32_t((uint64_t(a) + b - 1) / b); }

inline int column_vec(const Dims& d) { return (d.dtype == BNS_BF16 && d.C % 8 == 0) ? 8 : (d.C % 4 == 0) ? 4 : 1; }

// Blocks: enough to fill the device a few times over.  Reductions (blocks > 0, or the reduction
// default) keep at least four rows per row lane and a bounded number of partials per channel.
// split_bound (optional): the number of splits before the rows are dealt out evenly.  It never decreases when
// `rows` or `blocks` grow, and the final t.splits never exceeds it -- unlike t.splits itself, which the
// rounding of rows_per_block makes non-monotonic (924 rows -> 55 splits, 896 rows -> 56).
Tiling make_tiling(const Dims& d, uint32_t rows, int blocks = 0, bool elementwise = false,
                   uint32_t* split_bound = nullptr) {
    Tiling t;
    const int V = column_vec(d);
    t.C = d.C;
    t.CV = d.C / V;
    int l = 0;
    while ((1 << l) < t.CV && l < 6) ++l;
    t.log2_tx = l;
    const uint32_t tiles = uint32_t((t.CV + (1 << l) - 1) >> l);
    const uint32_t TY = uint32_t(kBlock >> l);
    uint32_t s;
    if (elementwise) {
        // short blocks of a few rows per row lane (the launch then streams through memory front to back
        // like a flat kernel); fewer rows per lane when that would leave compute units idle
        s = ceil_div_u(rows, TY * uint32_t(tuned(g_tuning.nhwc_ew_rows, kNhwcEwRows)));
        const uint32_t fill = ceil_div_u(uint32_t(kNhwcFill), tiles), cap = rows / TY;
        if (s < fill) s = fill < cap ? fill : cap;
    } else {
        if (blocks <= 0) blocks = tuned(g_tuning.nhwc_blocks, kNhwcBlocks);
        s = ceil_div_u(uint32_t(blocks), tiles);
        const uint32_t cap = rows / (TY * 4u);
        if (s > cap) s = cap;
        // a row lane adds its rows one after the other in fp32: keep that chain short
        const uint32_t lo = ceil_div_u(rows, TY * uint32_t(kNhwcMaxLaneRows));
        if (s < lo) s = lo;
        if (s > uint32_t(kNhwcMaxSplits)) s = kNhwcMaxSplits;
    }
    if (s < 1u) s = 1u;
    while (uint64_t(tiles) * s > 0x7FFFFFFFu) s = (s + 1u) / 2u;      // grid.x limit
    if (split_bound) *split_bound = s;
    t.rows_per_block = ceil_div_u(rows, s);
    t.splits = int32_t(ceil_div_u(rows, t.rows_per_block));     // no empty blocks
    return t;
}

inline uint32_t grid_of(const Tiling& t) {
    const uint32_t tiles = uint32_t((t.CV + (1 << t.log2_tx) - 1) >> t.log2_tx);
    return tiles * uint32_t(t.splits);
}

RowSet make_rowset(const Dims& d, const bns_box& b) {
    RowSet s;
    s.n0 = b.n0;
    s.h0 = b.h0;
    s.w0 = b.w0;
    s.H = d.H;
    s.W = d.W;
    s.patch_div = make_fastdiv(uint32_t(b.h_cnt) * uint32_t(b.w_cnt));
    s.pw_div = make_fastdiv(uint32_t(b.w_cnt));
    s.rows = uint32_t(b.n_cnt) * uint32_t(b.h_cnt) * uint32_t(b.w_cnt);
    s.pivot_rows = s.rows < uint32_t(kPivotRows) ? s.rows : uint32_t(kPivotRows);
    s.inv_pivot_rows = 1.0f / float(s.pivot_rows);
    s.contiguous = (b.w_cnt == d.W && (b.h_cnt == d.H || b.n_cnt == 1)) || (b.n_cnt == 1 && b.h_cnt == 1);
    return s;
}

RowBox make_rowbox(const Dims& d, const bns_box& b) {
    RowBox B;
    B.n0 = uint32_t(b.n0);
    B.n1 = uint32_t(b.n0 + b.n_cnt);
    B.h0 = uint32_t(b.h0);
    B.h1 = uint32_t(b.h0 + b.h_cnt);
    B.w0 = uint32_t(b.w0);
    B.w1 = uint32_t(b.w0 + b.w_cnt);
    B.hw_div = make_fastdiv(uint32_t(d.HW));
    B.w_div = make_fastdiv(uint32_t(d.W));
    return B;
}

// Tiling of the one-launch kernels: column lanes for 128 contiguous bytes of a row, every other lane
// on rows, one block per tile of channels.  False when a row lane would get more than kNhwcSmallRows.
bool small_tiling(const Dims& d, Tiling* t) {
    if (g_tuning.nhwc_small == 2) return false;
    const int V = column_vec(d);
    t->C = d.C;
    t->CV = d.C / V;
    const int want = 128 / (V * (d.dtype == BNS_F32 ? 4 : 2));
    int l = 0;
    while ((1 << l) < t->CV && (1 << l) < want) ++l;
    t->log2_tx = l;
    t->splits = 1;
    const uint32_t M = uint32_t(d.N) * uint32_t(d.HW);
    t->rows_per_block = M;
    const uint32_t TY = uint32_t(kBlock >> l);
    return ceil_div_u(M, TY) <= uint32_t(kNhwcSmallRows);
}

template <int V>
using VecTag = std::integral_constant<int, V>;

template <typename F>
hipError_t dispatch_nhwc(const Dims& d, F&& f) {
    const int V = column_vec(d);
    if (d.dtype == BNS_F32) return V == 4 ? f(float(), VecTag<4>()) : f(float(), VecTag<1>());
    if (V == 8) return f(bf16_t(), VecTag<8>());
    return V == 4 ? f(bf16_t(), VecTag<4>()) : f(bf16_t(), VecTag<1>());
}

template <typename T, int V>
hipError_t launch_stats_partial(const T* x, Partial* partial, const RowSet& S, const Tiling& t, hipStream_t st) {
    const dim3 grid(grid_of(t)), block(kBlock);
    // the normalization pass reads the rows of S again
    const bool keep = keep_for_next_pass(size_t(S.rows) * size_t(t.C) * sizeof(T));
    if (S.contiguous) {
        if (keep) BNS_LAUNCH((nhwc_stats_partial_kernel<T, V, true, true>), grid, block, 0, st, x, partial, S, t);
        else BNS_LAUNCH((nhwc_stats_partial_kernel<T, V, true, false>), grid, block, 0, st, x, partial, S, t);
    } else {
        if (keep) BNS_LAUNCH((nhwc_stats_partial_kernel<T, V, false, true>), grid, block, 0, st, x, partial, S, t);
        else BNS_LAUNCH((nhwc_stats_partial_kernel<T, V, false, false>), grid, block, 0, st, x, partial, S, t);
    }
    return hipGetLastError();
}

}  // namespace

size_t nhwc_partial_bytes(const Dims& d) {
    // the most splits make_tiling can choose for any row set of this shape and any block target
    uint32_t bound = 1;
    make_tiling(d, uint32_t(d.N) * uint32_t(d.HW), kNhwcBlocksMax, false, &bound);
    return (size_t(bound) * size_t(d.C) * sizeof(Partial) + 255) & ~size_t(255);
}

namespace {
// The partial sums of `t` must fit the workspace region the API sized with nhwc_partial_bytes.
inline bool fits_region(const Dims& d, const Tiling& t) {
    return size_t(t.splits) * size_t(d.C) * sizeof(Partial) <= nhwc_partial_bytes(d);
}
}  // namespace

hipError_t launch_nhwc_stats(const Dims& d, const bns_box& b, const void* x, Partial* partial, float eps, float momentum,
                             float* save_mean, float* save_invstd, float* running_mean, float* running_var,
                             hipStream_t st) {
    const RowSet S = make_rowset(d, b);
    const Tiling t = make_tiling(d, S.rows);
    if (!fits_region(d, t)) return hipErrorInvalidValue;
    return dispatch_nhwc(d, [&](auto ty, auto vt) {
        using T = decltype(ty);
        constexpr int V = decltype(vt)::value;
        hipError_t e = launch_stats_partial<T, V>(static_cast<const T*>(x), partial, S, t, st);
        if (e != hipSuccess) return e;
        BNS_LAUNCH((nhwc_stats_finalize_kernel<T>), dim3(ceil_div_u(uint32_t(d.C), kFinCh)), dim3(kBlock), 0, st,
                   static_cast<const T*>(x), partial, S, d.C, t.splits, eps, momentum, save_mean, save_invstd,
                   running_mean, running_var);
        return hipGetLastError();
    });
}

hipError_t launch_nhwc_normalize(const Dims& d, const void* x, const float* gamma, const float* beta, const float* mean,
                                 const float* invstd, void* y, hipStream_t st, float var_eps) {
    const uint32_t M = uint32_t(d.N) * uint32_t(d.HW);
    const Tiling t = make_tiling(d, M, 0, true);
    return dispatch_nhwc(d, [&](auto ty, auto vt) {
        using T = decltype(ty);
        constexpr int V = decltype(vt)::value;
        BNS_LAUNCH((nhwc_normalize_kernel<T, V>), dim3(grid_of(t)), dim3(kBlock), 0, st, static_cast<const T*>(x),
                   static_cast<T*>(y), gamma, beta, mean, invstd, t, M, var_eps);
        return hipGetLastError();
    });
}

hipError_t launch_nhwc_reduce(const Dims& d, const void* x, const void* dy, const float* mean, const float* invstd,
                              Partial* partial, float* dgamma, float* dbeta, bool x_again, hipStream_t st) {
    const uint32_t M = uint32_t(d.N) * uint32_t(d.HW);
    const Tiling t = make_tiling(d, M);
    if (!fits_region(d, t)) return hipErrorInvalidValue;
    // dy of as many row shares as fit is left in the memory-side cache for the dx pass (x too when that pass reads
    // most of it again and both fit)
    const size_t bytes = size_t(M) * size_t(d.C) * (d.dtype == BNS_F32 ? 4 : 2);
    const size_t share = size_t(t.rows_per_block) * size_t(d.C) * (d.dtype == BNS_F32 ? 4 : 2);
    const int reuse = g_tuning.cache_reuse;
    const uint32_t keep_splits =
        reuse == 2 ? 0u : reuse == 1 ? uint32_t(t.splits) : uint32_t(std::min<size_t>(size_t(t.splits), kKeepBytes / share));
    const int keep = keep_splits == 0u ? 0 : (x_again && keep_for_next_pass(2 * bytes)) ? 2 : 1;
    return dispatch_nhwc(d, [&](auto ty, auto vt) {
        using T = decltype(ty);
        constexpr int V = decltype(vt)::value;
        const dim3 grid(grid_of(t)), block(kBlock);
        const T* xp = static_cast<const T*>(x);
        const T* gp = static_cast<const T*>(dy);
        if (keep == 2) BNS_LAUNCH((nhwc_reduce_partial_kernel<T, V, 2>), grid, block, 0, st, xp, gp, mean, partial, t, M, keep_splits);
        else if (keep == 1) BNS_LAUNCH((nhwc_reduce_partial_kernel<T, V, 1>), grid, block, 0, st, xp, gp, mean, partial, t, M, keep_splits);
        else BNS_LAUNCH((nhwc_reduce_partial_kernel<T, V, 0>), grid, block, 0, st, xp, gp, mean, partial, t, M, keep_splits);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        BNS_LAUNCH(nhwc_reduce_finalize_kernel, dim3(ceil_div_u(uint32_t(d.C), kFinCh)), dim3(kBlock), 0, st,
                   partial, d.C, t.splits, invstd, dgamma, dbeta);
        return hipGetLastError();
    });
}

// The whole backward pass with dx split by Eq. 6's two branches: sums + dx outside S, finalize, dx on S.
hipError_t launch_nhwc_backward_split(const Dims& d, const bns_box& b, const void* x, const void* dy, const float* gamma,
                                      const float* mean, const float* invstd, Partial* partial, float* dgamma,
                                      float* dbeta, void* dx, hipStream_t st) {
    const uint32_t M = uint32_t(d.N) * uint32_t(d.HW);
    const Tiling t = make_tiling(d, M);      // the tiling of launch_nhwc_reduce: same partials, same sums, bit for bit
    if (!fits_region(d, t)) return hipErrorInvalidValue;
    const RowBox B = make_rowbox(d, b);
    const RowSet S = make_rowset(d, b);
    const Tiling ts = make_tiling(d, S.rows, 0, true);
    const double s = double(b.n_cnt) * double(b.h_cnt) * double(b.w_cnt);
    return dispatch_nhwc(d, [&](auto ty, auto vt) {
        using T = decltype(ty);
        constexpr int V = decltype(vt)::value;
        BNS_LAUNCH((nhwc_reduce_outside_kernel<T, V>), dim3(grid_of(t)), dim3(kBlock), 0, st,
                   static_cast<const T*>(x), static_cast<const T*>(dy), mean, partial, t, M, static_cast<T*>(dx), gamma,
                   invstd, B);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        BNS_LAUNCH(nhwc_reduce_finalize_kernel, dim3(ceil_div_u(uint32_t(d.C), kFinCh)), dim3(kBlock), 0, st,
                   partial, d.C, t.splits, invstd, dgamma, dbeta);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (S.contiguous)
            BNS_LAUNCH((nhwc_dx_rows_kernel<T, V, true>), dim3(grid_of(ts)), dim3(kBlock), 0, st, static_cast<const T*>(x),
                       static_cast<const T*>(dy), static_cast<T*>(dx), gamma, mean, invstd, dgamma, dbeta, S, ts,
                       float(1.0 / s));
        else
            BNS_LAUNCH((nhwc_dx_rows_kernel<T, V, false>), dim3(grid_of(ts)), dim3(kBlock), 0, st, static_cast<const T*>(x),
                       static_cast<const T*>(dy), static_cast<T*>(dx), gamma, mean, invstd, dgamma, dbeta, S, ts,
                       float(1.0 / s));
        return hipGetLastError();
    });
}

hipError_t launch_nhwc_dx(const Dims& d, const bns_box& b, const void* x, const void* dy, const float* gamma,
                          const float* mean, const float* invstd, const float* dgamma, const float* dbeta, void* dx,
                          hipStream_t st) {
    const uint32_t M = uint32_t(d.N) * uint32_t(d.HW);
    const Tiling t = make_tiling(d, M, 0, true);
    const RowBox B = make_rowbox(d, b);
    const double s = double(b.n_cnt) * double(b.h_cnt) * double(b.w_cnt);
    return dispatch_nhwc(d, [&](auto ty, auto vt) {
        using T = decltype(ty);
        constexpr int V = decltype(vt)::value;
        BNS_LAUNCH((nhwc_dx_kernel<T, V>), dim3(grid_of(t)), dim3(kBlock), 0, st, static_cast<const T*>(x),
                   static_cast<const T*>(dy), static_cast<T*>(dx), gamma, mean, invstd, dgamma, dbeta, B, t, M,
                   float(1.0 / s));
        return hipGetLastError();
    });
}

bool launch_nhwc_small_forward(const Dims& d, const bns_box& b, const void* x, const float* gamma, const float* beta,
                               float eps, float momentum, void* y, float* save_mean, float* save_invstd,
                               float* running_mean, float* running_var, hipStream_t st, hipError_t* err) {
    Tiling t;
    if (!small_tiling(d, &t)) return false;
    const RowSet S = make_rowset(d, b);
    const uint32_t M = uint32_t(d.N) * uint32_t(d.HW);
    *err = dispatch_nhwc(d, [&](auto ty, auto vt) {
        using T = decltype(ty);
        constexpr int V = decltype(vt)::value;
        BNS_LAUNCH((nhwc_small_forward_kernel<T, V>), dim3(grid_of(t)), dim3(kBlock), 0, st,
                   static_cast<const T*>(x), static_cast<T*>(y), gamma, beta, S, t, M, eps, momentum, save_mean,
                   save_invstd, running_mean, running_var);
        return hipGetLastError();
    });
    return true;
}

bool launch_nhwc_small_backward(const Dims& d, const bns_box& b, const void* x, const void* dy, const float* gamma,
                                const float* mean, const float* invstd, void* dx, float* dgamma, float* dbeta,
                                hipStream_t st, hipError_t* err) {
    Tiling t;
    if (!small_tiling(d, &t)) return false;
    const RowBox B = make_rowbox(d, b);
    const uint32_t M = uint32_t(d.N) * uint32_t(d.HW);
    const double s = double(b.n_cnt) * double(b.h_cnt) * double(b.w_cnt);
    *err = dispatch_nhwc(d, [&](auto ty, auto vt) {
        using T = decltype(ty);
        constexpr int V = decltype(vt)::value;
        BNS_LAUNCH((nhwc_small_backward_kernel<T, V>), dim3(grid_of(t)), dim3(kBlock), 0, st,
                   static_cast<const T*>(x), static_cast<const T*>(dy), static_cast<T*>(dx), gamma, mean, invstd,
                   dgamma, dbeta, B, t, M, float(1.0 / s));
        return hipGetLastError();
    });
    return true;
}

// Eq. 4 forward statistics: `partial` holds two regions of nhwc_partial_bytes(d) each (set S, then set V).
hipError_t launch_nhwc_stats_mixed(const Dims& d, const bns_box& b, int n_v, const void* x, Partial* partial,
                                   float mix_beta, float eps, float momentum, float* save_mean, float* save_invstd,
                                   float* mean_parts, float* running_mean, float* running_var, hipStream_t st) {
    const RowSet S = make_rowset(d, b);
    const bns_box vb{0, n_v, 0, d.H, 0, d.W};
    const RowSet Vs = make_rowset(d, vb);
    const Tiling ts = make_tiling(d, S.rows), tv = make_tiling(d, Vs.rows);
    if (!fits_region(d, ts) || !fits_region(d, tv)) return hipErrorInvalidValue;
    Partial* partial_v = reinterpret_cast<Partial*>(reinterpret_cast<char*>(partial) + nhwc_partial_bytes(d));
    return dispatch_nhwc(d, [&](auto ty, auto vt) {
        using T = decltype(ty);
        constexpr int V = decltype(vt)::value;
        hipError_t e = launch_stats_partial<T, V>(static_cast<const T*>(x), partial, S, ts, st);
        if (e != hipSuccess) return e;
        if ((e = launch_stats_partial<T, V>(static_cast<const T*>(x), partial_v, Vs, tv, st)) != hipSuccess) return e;
        BNS_LAUNCH((nhwc_stats_finalize_mixed_kernel<T>), dim3(ceil_div_u(uint32_t(d.C), kFinCh)), dim3(kBlock), 0,
                   st, static_cast<const T*>(x), partial, ts.splits, partial_v, tv.splits, S, Vs, d.C, mix_beta, eps,
                   momentum, save_mean, save_invstd, mean_parts, running_mean, running_var);
        return hipGetLastError();
    });
}

hipError_t launch_nhwc_dx_mixed(const Dims& d, const bns_box& b, int n_v, float mix_beta, const void* x, const void* dy,
                                const float* gamma, const float* invstd, const float* dgamma, const float* dbeta,
                                const float* mean_parts, void* dx, hipStream_t st) {
    const uint32_t M = uint32_t(d.N) * uint32_t(d.HW);
    const Tiling t = make_tiling(d, M, 0, true);
    const RowBox B = make_rowbox(d, b);
    const float w_s = float((1.0 - double(mix_beta)) / (double(b.n_cnt) * double(b.h_cnt) * double(b.w_cnt)));
    const float w_v = float(double(mix_beta) / (double(n_v) * double(d.HW)));
    return dispatch_nhwc(d, [&](auto ty, auto vt) {
        using T = decltype(ty);
        constexpr int V = decltype(vt)::value;
        BNS_LAUNCH((nhwc_dx_mixed_kernel<T, V>), dim3(grid_of(t)), dim3(kBlock), 0, st, static_cast<const T*>(x),
                   static_cast<const T*>(dy), static_cast<T*>(dx), gamma, invstd, dgamma, dbeta, mean_parts,
                   mean_parts + d.C, B, uint32_t(n_v) * uint32_t(d.HW), w_v, w_s, t, M);
        return hipGetLastError();
    });
}

}  // namespace bns
