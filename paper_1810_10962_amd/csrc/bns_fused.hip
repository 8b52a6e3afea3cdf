// Fused single-launch kernels: a channel stays on chip between its reduction and its
// element-wise pass.
//
// The paper counts the cost of BN in reductions over m points followed by a second pass
// over the same data (Sec. 3.1, Fig. 1c/d).  On MI355X a channel of a typical layer
// (0.1 - 1 MB) fits in the vector registers of one or a few compute units (512 KB each),
// so the second pass need not touch HBM again:
//
//   forward : read x once, keep it in registers, statistics over S (Eq. 3), normalise
//             (Eq. 1), write y                               ->  2e bytes per element
//   backward: read dy (kept in registers) and x once, sums over all m (Eq. 5), then
//             dx (Eq. 6) re-reading x only on S              ->  (3 + r)e bytes per element
//
// A *team* of T blocks owns one channel at a time; each member keeps 1/T of the channel's
// vectors in registers (KMAX 16-byte vectors per thread).  Members exchange their partial
// sums through stamped slots in the workspace (an all-gather): each slot word is a 64-bit
// value {payload float, 32-bit stamp} written and polled with relaxed agent-scope atomics,
// so payload and stamp always arrive together and no slot has to be cleared beforehand.
// Every member adds the T partials in member order, so all members get bit-identical
// statistics, and results do not depend on timing.
//
// Waiting on a team-mate is safe because the grid never exceeds what the device holds at once
// (occupancy query x compute units) and because the blocks of a team have consecutive indices and
// blocks are started in index order: a team-mate that is not running yet is next in line for a
// slot, and slots are freed by complete teams, which depend on nothing else.  The wait is bounded
// all the same: if a team-mate's slot never arrives, the sums become NaN and the kernel still
// runs to completion.
#include <hip/hip_runtime.h>

#include <atomic>
#include <chrono>
#include <mutex>

#include "bns_device.hpp"
#include "bns_fused_device.hpp"
#include "bns_internal.hpp"

namespace bns {

namespace {

// ---------------------------------------------------------------------------------------
// Forward: Eq. 3 + Eq. 8 + Eq. 1 with x read once
// ---------------------------------------------------------------------------------------
// PATCH: S is a patch of each plane (host guarantee: h_cnt * w_cnt < H * W); else (0) S is whole planes.
//   1: the sampled elements are read on their own, ahead of the vectors (see below);
//   2: the statistics are taken from the vectors in the registers under a per-row column mask -- for a block
//      that holds its channel alone (T = 1, nothing to exchange while the vectors arrive) and rows that are a
//      whole number of vectors; it then costs what full BN costs instead of a second, scattered read.
// MIXED: Eq. 4 -- a second pair of sums over the virtual set (samples [0, n_v), always whole planes, taken
// from the registers), a second exchange, and the blend of the two (E, Var) pairs.
// Eq. 4 at (512 threads, up to 16 vectors) runs two blocks per compute unit, i.e. four waves per SIMD and at most 128
// registers; the compiler is told so, because left alone it takes 150 and the second block is gone (130x128x28x28,
// 7x7 patch + 2 virtual samples: forward 34 -> 29.7 us, a few registers spilled included).
template <typename T, int V, int KMAX, int NT, int PATCH, bool MIXED>
__global__ __launch_bounds__(NT, (MIXED && NT == 512 && KMAX <= 16) ? 4 : 1) void fused_forward_kernel(FusedArgs A) {
    typedef RawVec<T, V> RV;
    __shared__ float red[2 * (NT / kWave)];
    __shared__ float team_lds[2 * kMaxTeam];
    __shared__ double bc[2];
    __shared__ uint32_t words[3];                           // launch stamp, flags of the exchanges
    const int team = blockIdx.x / A.T;
    if (team >= A.num_teams) return;                       // blocks beyond the last whole team
    const int j = blockIdx.x - team * A.T;
    const uint32_t hwv = A.hwv_div.d;
    // Member j owns the NT-vector chunks j, j + T, j + 2T, ... of the channel (round-robin, so that
    // every member sees the same mix of sampled and unsampled planes and finishes at the same time).
    const uint32_t beg = uint32_t(j) * NT;
    const uint32_t step = uint32_t(A.T) * NT;
    const uint32_t end = A.tot;
    const size_t nstride = size_t(A.C) * A.HW;
    const T* x = static_cast<const T*>(A.x);
    T* y = static_cast<T*>(A.out);

    // The launch stamp (every block of the grid reads the workspace header once): behind the first channel's loads,
    // where the round trip costs nothing -- except in the variants that fill the register file with that channel,
    // which take it first (they run with one or few blocks per channel, where a microsecond at the start is cheap
    // and spilled registers are not).
    constexpr bool kStampFirst = KMAX >= 32;
    if (kStampFirst) stamp_accept(A, stamp_request(A), words);

    uint32_t it = 0;
    for (int cl = team; cl < A.cg; cl += A.num_teams, ++it) {
        const int c = A.c0 + cl;
        const bns_box b = box_of_channel(A.ip, c);
        const T* xc = x + size_t(c) * A.HW;
        T* yc = y + size_t(c) * A.HW;
        const T* first = xc + size_t(b.n0) * nstride + size_t(b.h0) * A.W + b.w0;       // first sampled element
        const float pivot = load_scalar<T>(first);

        // A patch of each plane (Feature Sampling): the sampled elements are few and scattered inside the
        // vectors, so they are read on their own, element q = (n, ph, pw) by thread q mod (T * NT), BEFORE the
        // vectors of the channel.  Loads return in order, so the statistics and the exchange then run while
        // the vectors are still on their way, and no vector has to be masked element by element.
        constexpr int kPatchLoads = patch_loads(KMAX, MIXED);
        float pe[PATCH == 1 ? kPatchLoads : 1];
        const uint32_t q0 = uint32_t(j) * NT + threadIdx.x;
        if constexpr (PATCH == 1) {
#pragma unroll
            for (int m = 0; m < kPatchLoads; ++m) {
                const uint32_t q = q0 + uint32_t(m) * step;
                pe[m] = q < A.s_cnt ? load_scalar<T>(first + patch_offset(A, q, nstride)) : pivot;
            }
        }

        typename RV::raw_t v[KMAX];
        const uint32_t ia = opaque(beg + threadIdx.x);
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const uint32_t i = ia + uint32_t(k) * step;
            if (i < end) {
                const uint32_t n = fdiv(i, A.hwv_div);
                v[k] = RV::ld(xc + n * nstride + size_t(i - n * hwv) * V);
            }
        }
        float s1 = 0.f, s2 = 0.f;
        if constexpr (PATCH == 2) {                                 // rows h0 .. h1-1, columns w0 .. w1-1 of every vector row
            static_assert(KMAX <= 64, "one bit per vector");
            const uint32_t wvr = A.wv_div.d;                        // vectors per row
            const uint32_t wv0 = uint32_t(b.w0) / V;                // vector columns that touch the patch
            const uint32_t nvw = uint32_t(b.w0 + b.w_cnt - 1) / V - wv0 + 1u;
            if (A.patch_stage) {
                // The block holds the whole channel.  A use of a loaded vector inside a divergent branch makes the
                // compiler wait for every load, so masking the vectors where they sit would put all of that
                // arithmetic behind the last load.  Instead: which vectors touch the patch is worked out while the
                // loads are in flight (it needs no data); those few are then copied to LDS, vector (n, h, column)
                // to a slot of its own, and every thread takes its share of the slots -- dense work, the same
                // order of additions in every run.
                __shared__ typename RV::raw_t stage[kStageSlots];
                const uint32_t ib = opaque(beg + threadIdx.x);
                unsigned long long hits = 0;
#pragma unroll
                for (int k = 0; k < KMAX; ++k) {
                    const uint32_t i = ib + uint32_t(k) * step;
                    const uint32_t n = fdiv(i, A.hwv_div);
                    const uint32_t rem = i - n * hwv;
                    const uint32_t h = fdiv(rem, A.wv_div);
                    const uint32_t wc = rem - h * wvr;
                    const bool in = i < end && n - uint32_t(b.n0) < uint32_t(b.n_cnt) && h - uint32_t(b.h0) < uint32_t(b.h_cnt) &&
                                    wc - wv0 < nvw;
                    hits |= (unsigned long long)(in) << k;
                }
#pragma unroll
                for (int k = 0; k < KMAX; ++k) {
                    if ((hits >> k) & 1ull) {
                        const uint32_t i = ib + uint32_t(k) * step;
                        const uint32_t n = fdiv(i, A.hwv_div);
                        const uint32_t rem = i - n * hwv;
                        const uint32_t h = fdiv(rem, A.wv_div);
                        const uint32_t wc = rem - h * wvr;
                        stage[((n - uint32_t(b.n0)) * uint32_t(b.h_cnt) + (h - uint32_t(b.h0))) * nvw + (wc - wv0)] = v[k];
                    }
                }
                __syncthreads();
                const uint32_t slots = uint32_t(b.n_cnt) * uint32_t(b.h_cnt) * nvw;
                uint32_t wc = threadIdx.x % nvw;                    // column of slot q = q mod nvw, carried along
                const uint32_t wstep = NT % nvw;
                for (uint32_t q = threadIdx.x; q < slots; q += NT) {
                    const int32_t col = int32_t(wv0 + wc) * V;
                    const int32_t lo = max(b.w0 - col, 0), hi = min(b.w0 + b.w_cnt - col, V);
                    float f[V];
                    RV::unpack(stage[q], f);
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        const float d = (e >= lo && e < hi) ? f[e] - pivot : 0.f;
                        s1 += d;
                        s2 = fmaf(d, d, s2);
                    }
                    wc += wstep;
                    if (wc >= nvw) wc -= nvw;
                }
            } else {
                const uint32_t ib = opaque(beg + threadIdx.x);
#pragma unroll
                for (int k = 0; k < KMAX; ++k) {
                    const uint32_t i = ib + uint32_t(k) * step;
                    if (i < end) {
                        const uint32_t n = fdiv(i, A.hwv_div);
                        const uint32_t rem = i - n * hwv;
                        const uint32_t h = fdiv(rem, A.wv_div);
                        const int32_t col = int32_t(rem - h * wvr) * V;         // first column of the vector
                        const int32_t lo = max(b.w0 - col, 0), hi = min(b.w0 + b.w_cnt - col, V);
                        if (n - uint32_t(b.n0) < uint32_t(b.n_cnt) && h - uint32_t(b.h0) < uint32_t(b.h_cnt) && lo < hi) {
                            float f[V];
                            RV::unpack(v[k], f);
#pragma unroll
                            for (int e = 0; e < V; ++e) {
                                const float d = (e >= lo && e < hi) ? f[e] - pivot : 0.f;
                                s1 += d;
                                s2 = fmaf(d, d, s2);
                            }
                        }
                    }
                }
            }
        } else if constexpr (!PATCH) {                              // whole planes of some samples: from the registers
            const uint32_t ib = opaque(beg + threadIdx.x);
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                const uint32_t i = ib + uint32_t(k) * step;
                if (i < end) {
                    const uint32_t n = fdiv(i, A.hwv_div);
                    if (n >= uint32_t(b.n0) && n < uint32_t(b.n0 + b.n_cnt)) {
                        float f[V];
                        RV::unpack(v[k], f);
#pragma unroll
                        for (int e = 0; e < V; ++e) {
                            const float d = f[e] - pivot;
                            s1 += d;
                            s2 = fmaf(d, d, s2);
                        }
                    }
                }
            }
        } else {
#pragma unroll
            for (int m = 0; m < kPatchLoads; ++m) {                 // padded with the pivot: d = 0
                const float d = pe[m] - pivot;
                s1 += d;
                s2 = fmaf(d, d, s2);
            }
            // what is left of the patch (most of it when one block holds the channel), a few loads in flight at a time
            constexpr int kBatch = KMAX >= 50 ? 2 : KMAX >= 32 ? 4 : KMAX >= 16 ? 1 : 8;      // (registers)
            for (uint32_t q = q0 + uint32_t(kPatchLoads) * step; q < A.s_cnt; q += uint32_t(kBatch) * step) {
                float t[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const uint32_t qu = q + uint32_t(u) * step;
                    t[u] = qu < A.s_cnt ? load_scalar<T>(first + patch_offset(A, qu, nstride)) : pivot;
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const float d = t[u] - pivot;
                    s1 += d;
                    s2 = fmaf(d, d, s2);
                }
            }
        }
        float v1 = 0.f, v2 = 0.f, pivot_v = 0.f;
        if constexpr (MIXED) {                                      // the virtual set: planes of samples [0, n_v)
            pivot_v = load_scalar<T>(xc);
            const uint32_t id = opaque(beg + threadIdx.x);
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                const uint32_t i = id + uint32_t(k) * step;
                if (i < end && fdiv(i, A.hwv_div) < uint32_t(A.n_v)) {
                    float f[V];
                    RV::unpack(v[k], f);
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        const float d = f[e] - pivot_v;
                        v1 += d;
                        v2 = fmaf(d, d, v2);
                    }
                }
            }
        }
        if (!kStampFirst && it == 0) stamp_accept(A, stamp_request(A), words);
        block_allsum2<NT>(s1, s2, red);
        if (NT == kWave) __syncthreads();                       // (one wave: block_allsum2 has no barrier of its own)
        double t1, t2;
        bool arrived = team_allsum2<NT>(A, words, team * A.T, j, MIXED ? 2u * it : it, s1, s2, t1, t2, team_lds, bc);

        // Eq. 3 (every thread computes the same values from the same totals)
        const double m1 = t1 / A.s;
        double mean = double(pivot) + m1;
        double var = t2 / A.s - m1 * m1;
        if (!(var >= 0.0)) var = (var != var) ? var : 0.0;      // clamp rounding; keep NaN visible
        if constexpr (MIXED) {
            __syncthreads();                                    // red[] is read by every thread of the first sum
            block_allsum2<NT>(v1, v2, red);
            double u1, u2;
            arrived &= team_allsum2<NT>(A, words, team * A.T, j, 2u * it + 1u, v1, v2, u1, u2, team_lds, bc);
            const double mv = u1 / A.s_v;
            const double e_v = double(pivot_v) + mv;
            double var_v = u2 / A.s_v - mv * mv;
            if (!(var_v >= 0.0)) var_v = (var_v != var_v) ? var_v : 0.0;
            if (j == 0 && threadIdx.x == 0) {
                A.mean_parts[c] = float(e_v);
                A.mean_parts[A.C + c] = float(mean);
            }
            const double bm = double(A.mix_beta);
            mean = bm * e_v + (1.0 - bm) * mean;                // Eq. 4, X = E
            var = bm * var_v + (1.0 - bm) * var;                // Eq. 4, X = Var
        }
        const float mu = float(mean);
        const float r = float(1.0 / sqrt(var + double(A.eps)));
        if (j == 0 && threadIdx.x == 0) {
            A.save_mean[c] = mu;
            A.save_invstd[c] = r;
            const double al = double(A.momentum);
            // (a wait for a team-mate that ran out leaves NaN statistics; the moving averages then stay as they are)
            if (A.running_mean && arrived) A.running_mean[c] = float((1.0 - al) * double(A.running_mean[c]) + al * mean);
            if (A.running_var && arrived) A.running_var[c] = float((1.0 - al) * double(A.running_var[c]) + al * var);
        }
        const float sc = settled(A.gamma[c]) * r;
        const float sh = settled(A.beta[c]);
        const uint32_t ic = opaque(beg + threadIdx.x);
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const uint32_t i = ic + uint32_t(k) * step;
            if (i < end) {
                const uint32_t n = fdiv(i, A.hwv_div);
                float f[V];
                opaque_raw(v[k]);
                RV::unpack(v[k], f);
#pragma unroll
                for (int e = 0; e < V; ++e) f[e] = fmaf(f[e] - mu, sc, sh);
                RV::st(yc + n * nstride + size_t(i - n * hwv) * V, RV::pack(f));
            }
        }
    }
    team_done(A, j, read_stamp(A, words));
}

// ---------------------------------------------------------------------------------------
// Backward: Eq. 5 sums + Eq. 6 with dy read once
// ---------------------------------------------------------------------------------------
// KEEPX: x stays in registers next to dy (KMAX vectors of each), so nothing is read twice; worth its
// registers when most of the channel lies in S (full BN).
// MIXED: backward of Eq. 4 -- vectors of samples [0, n_v) belong to the virtual set (weight w_v, centre E_v,
// every element), vectors that touch the box to the sampled real set (w_s, centre E_s, masked by the box).
template <typename T, int V, int KMAX, int NT, bool KEEPX, bool MIXED>
__global__ __launch_bounds__(NT, (KEEPX && NT == 512 && KMAX <= 8) ? 4 : 1) void fused_backward_kernel(FusedArgs A) {
    typedef RawVec<T, V> RV;
    __shared__ float red[2 * (NT / kWave)];
    __shared__ float team_lds[2 * kMaxTeam];
    __shared__ double bc[2];
    __shared__ uint32_t words[3];                           // launch stamp, flags of the exchanges
    const int team = blockIdx.x / A.T;
    if (team >= A.num_teams) return;
    const int j = blockIdx.x - team * A.T;
    const uint32_t hwv = A.hwv_div.d;
    const uint32_t beg = uint32_t(j) * NT;                    // chunks j, j + T, ... as in the forward kernel
    const uint32_t step = uint32_t(A.T) * NT;
    const uint32_t end = A.tot;
    const size_t nstride = size_t(A.C) * A.HW;
    const T* x = static_cast<const T*>(A.x);
    const T* dy = static_cast<const T*>(A.dy);
    T* dx = static_cast<T*>(A.out);

    constexpr bool kStampFirst = KMAX >= 32;               // as in the forward kernel
    if (kStampFirst) stamp_accept(A, stamp_request(A), words);

    uint32_t it = 0;
    for (int cl = team; cl < A.cg; cl += A.num_teams, ++it) {
        const int c = A.c0 + cl;
        const bns_box b = box_of_channel(A.ip, c);
        const T* xc = x + size_t(c) * A.HW;
        const T* gc = dy + size_t(c) * A.HW;
        T* dc = dx + size_t(c) * A.HW;
        const float mu = settled(A.save_mean[c]);
        const float r = settled(A.save_invstd[c]);
        const float ga = settled(A.gamma[c]);

        typename RV::raw_t g[KMAX];
        const uint32_t ia = opaque(beg + threadIdx.x);
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const uint32_t i = ia + uint32_t(k) * step;
            if (i < end) {
                const uint32_t n = fdiv(i, A.hwv_div);
                g[k] = RV::ld(gc + n * nstride + size_t(i - n * hwv) * V);
            }
        }
        float s1 = 0.f, s2 = 0.f;
        typename RV::raw_t xk[KEEPX ? KMAX : 1];
        constexpr int XB = (KMAX >= 50 || (V == 8 && KMAX > 16)) ? 2 : 4;        // x vectors in flight per thread (register budget)
        const uint32_t ib = opaque(beg + threadIdx.x);
        if constexpr (KEEPX) {
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                const uint32_t i = ib + uint32_t(k) * step;
                if (i < end) {
                    const uint32_t n = fdiv(i, A.hwv_div);
                    xk[k] = RV::ld(xc + n * nstride + size_t(i - n * hwv) * V);
                }
            }
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                const uint32_t i = ib + uint32_t(k) * step;
                if (i < end) {
                    float fg[V], fx[V];
                    RV::unpack(g[k], fg);
                    RV::unpack(xk[k], fx);
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        s1 += fg[e];
                        s2 = fmaf(fg[e], fx[e] - mu, s2);
                    }
                }
            }
        } else {
#pragma unroll
        for (int k0 = 0; k0 < KMAX; k0 += XB) {
            typename RV::raw_t xv[XB];
#pragma unroll
            for (int u = 0; u < XB; ++u) {
                const uint32_t i = ib + uint32_t(k0 + u) * step;
                if (k0 + u < KMAX && i < end) {
                    const uint32_t n = fdiv(i, A.hwv_div);
                    xv[u] = RV::ld(xc + n * nstride + size_t(i - n * hwv) * V);
                }
            }
#pragma unroll
            for (int u = 0; u < XB; ++u) {
                const uint32_t i = ib + uint32_t(k0 + u) * step;
                if (k0 + u < KMAX && i < end) {
                    float fg[V], fx[V];
                    RV::unpack(g[k0 + u < KMAX ? k0 + u : 0], fg);
                    RV::unpack(xv[u], fx);
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        s1 += fg[e];
                        s2 = fmaf(fg[e], fx[e] - mu, s2);
                    }
                }
            }
        }
        }
        if (!kStampFirst && it == 0) stamp_accept(A, stamp_request(A), words);
        block_allsum2<NT>(s1, s2, red);
        if (NT == kWave) __syncthreads();
        double t1, t2;
        team_allsum2<NT>(A, words, team * A.T, j, it, s1, s2, t1, t2, team_lds, bc);

        const float dbeta = float(t1);
        const float dgamma = float(t2 * double(r));
        if (j == 0 && threadIdx.x == 0) {
            A.dbeta[c] = dbeta;
            A.dgamma[c] = dgamma;
        }
        const float a = ga * r;
        const float wgt_s = MIXED ? A.w_s : A.inv_s;
        const float k1 = a * wgt_s * dbeta;
        const float k2 = a * wgt_s * dgamma * r;
        const float k1v = MIXED ? a * A.w_v * dbeta : 0.f;
        const float k2v = MIXED ? a * A.w_v * dgamma * r : 0.f;
        const float centre_s = MIXED ? A.mean_parts[A.C + c] : mu;
        const float centre_v = MIXED ? A.mean_parts[c] : mu;
        const uint32_t ic = opaque(beg + threadIdx.x);
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const uint32_t i = ic + uint32_t(k) * step;
            if (i < end) {
                const uint32_t n = fdiv(i, A.hwv_div);
                const uint32_t off = i - n * hwv;
                const uint32_t e0 = off * V;
                float f[V];
                opaque_raw(g[k]);
                RV::unpack(g[k], f);
                const bool virt = MIXED && n < uint32_t(A.n_v);
                const bool touches = virt || (n >= uint32_t(b.n0) && n < uint32_t(b.n0 + b.n_cnt) &&
                                              e0 + V > uint32_t(b.h0) * A.W && e0 < uint32_t(b.h0 + b.h_cnt) * A.W);
                if (touches) {
                    float fx[V];
                    if constexpr (KEEPX) {
                        opaque_raw(xk[k]);
                        RV::unpack(xk[k], fx);
                    } else {
                        RV::unpack(RV::ld(xc + n * nstride + size_t(off) * V), fx);
                    }
                    uint32_t h = fdiv(e0, A.w_div);
                    uint32_t w = e0 - h * uint32_t(A.W);
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        const float corr = virt             ? fmaf(k2v, fx[e] - centre_v, k1v)
                                           : in_hw(b, h, w) ? fmaf(k2, fx[e] - centre_s, k1)
                                                            : 0.f;
                        f[e] = fmaf(a, f[e], -corr);
                        if (++w == uint32_t(A.W)) {
                            w = 0;
                            ++h;
                        }
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < V; ++e) f[e] *= a;
                }
                RV::st(dc + n * nstride + size_t(off) * V, RV::pack(f));
            }
        }
    }
    team_done(A, j, read_stamp(A, words));
}

// ---------------------------------------------------------------------------------------
// Host side: choice of block size, registers per thread and team size
// ---------------------------------------------------------------------------------------
struct Variant {
    int nt, kmax;
};
// (threads per block, 16-byte vectors per thread).  Registers grow with kmax, so small
// channels take small variants and several blocks share a compute unit.
constexpr Variant kVariants[] = {{64, 1}, {128, 2}, {256, 4}, {512, 8}, {512, 16}, {512, 32}, {512, 50}};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

// Kernel kind = backward | flavour << 1 | mixed << 2.  Flavour: forward, statistics from separately read
// patch elements; backward, x kept in registers (built for the variants of up to kKeepXMaxVectors vectors
// per tensor only: beyond, the registers run out).  Mixed: Eq. 4 (built for vector accesses and up to
// kMixedMaxVectors vectors per thread; other shapes take the streaming kernels).
constexpr int kKeepXMaxVectors = 8;
constexpr int kMixedMaxVectors = 16;
template <typename T, int V>
const void* kernel_ptr(int kind, int variant) {
#define BNS_CASE(I, NT_, K_)                                                                                  \
    case I:                                                                                                   \
        if (kind == 3) {                                                                                      \
            if constexpr (K_ <= kKeepXMaxVectors)                                                             \
                return reinterpret_cast<const void*>(&fused_backward_kernel<T, V, K_, NT_, true, false>);     \
            else                                                                                              \
                return nullptr;                                                                               \
        }                                                                                                     \
        if (kind >= 4) {                                                                                      \
            if constexpr (K_ <= kMixedMaxVectors && V > 1) {                                                  \
                if (kind == 7) {                                                                              \
                    if constexpr (K_ <= kKeepXMaxVectors)                                                     \
                        return reinterpret_cast<const void*>(&fused_backward_kernel<T, V, K_, NT_, true, true>); \
                    else                                                                                      \
                        return nullptr;                                                                       \
                }                                                                                             \
                return kind == 5   ? reinterpret_cast<const void*>(&fused_backward_kernel<T, V, K_, NT_, false, true>) \
                       : kind == 6 ? reinterpret_cast<const void*>(&fused_forward_kernel<T, V, K_, NT_, 1, true>)   \
                                   : reinterpret_cast<const void*>(&fused_forward_kernel<T, V, K_, NT_, 0, true>); \
            } else {                                                                                          \
                return nullptr;                                                                               \
            }                                                                                                 \
        }                                                                                                     \
        return kind == 1   ? reinterpret_cast<const void*>(&fused_backward_kernel<T, V, K_, NT_, false, false>) \
               : kind == 2 ? reinterpret_cast<const void*>(&fused_forward_kernel<T, V, K_, NT_, 1, false>)   \
                           : reinterpret_cast<const void*>(&fused_forward_kernel<T, V, K_, NT_, 0, false>);
    switch (variant) {
        BNS_CASE(0, 64, 1)
        BNS_CASE(1, 128, 2)
        BNS_CASE(2, 256, 4)
        BNS_CASE(3, 512, 8)
        BNS_CASE(4, 512, 16)
        BNS_CASE(5, 512, 32)
        BNS_CASE(6, 512, 50)
    }
#undef BNS_CASE
    return nullptr;
}

const void* kernel_for(const Dims& d, int kind, int variant) {
    if (d.dtype == BNS_F32) return d.vec == 4 ? kernel_ptr<float, 4>(kind, variant) : kernel_ptr<float, 1>(kind, variant);
    if (d.vec == 8) return kernel_ptr<bf16_t, 8>(kind, variant);
    if (d.vec == 4) return kernel_ptr<bf16_t, 4>(kind, variant);
    return kernel_ptr<bf16_t, 1>(kind, variant);
}

// Forward, S a patch, statistics from the registers under a column mask (PATCH = 2): built for the two variants
// that hold a 64x56x56 channel in one block.
constexpr int kMaskedFirstVariant = 5;
const void* masked_forward_kernel(const Dims& d, int variant) {
    if (d.vec == 1 || d.W % d.vec != 0) return nullptr;
#define BNS_MASKED(T, V)                                                                               \
    return variant == 5   ? reinterpret_cast<const void*>(&fused_forward_kernel<T, V, 32, 512, 2, false>) \
           : variant == 6 ? reinterpret_cast<const void*>(&fused_forward_kernel<T, V, 50, 512, 2, false>) \
                          : nullptr;
    if (d.dtype == BNS_F32) {
        BNS_MASKED(float, 4)
    }
    if (d.vec == 8) {
        BNS_MASKED(bf16_t, 8)
    }
    BNS_MASKED(bf16_t, 4)
#undef BNS_MASKED
}

constexpr int kMaxPipeVariants = 16;
struct DeviceInfo {
    int cus = 0;
    int coop = 0;
    int blocks_per_cu[8][5][kNumVariants];  // [kernel kind][type/vec combo][variant], 0 = not queried yet
    int pipe_blocks_per_cu[5][kMaxPipeVariants];
    hipEvent_t chain_event = nullptr;       // orders launches whose blocks wait for each other across streams
    hipStream_t chain_stream = nullptr;     // the stream the last such launch went to
    bool chain_active = false;
};
DeviceInfo g_dev[16];
std::mutex g_dev_mutex;   // guards g_dev: launches may come from several host threads

int combo_index(const Dims& d) {
    if (d.dtype == BNS_F32) return d.vec == 4 ? 0 : 1;
    return d.vec == 8 ? 2 : d.vec == 4 ? 3 : 4;
}

// Exchange stamps count up from a start drawn when the library is loaded: a workspace whose memory still holds the
// slots of an earlier instance of the library in the same process (unloaded and loaded again) then does not meet its
// old stamps again.
uint32_t first_stamp() {
    uint64_t z = uint64_t(std::chrono::steady_clock::now().time_since_epoch().count()) ^
                 (uint64_t(reinterpret_cast<uintptr_t>(&g_dev)) << 17);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return uint32_t(z >> 32) | 1u;
}
std::atomic<uint32_t> g_stamp{first_stamp()};

}  // namespace

// bns_fused_pipe.hip
int pipe_variant_count();
int pipe_default_variant(const Dims& d);
int pipe_alternative_variant(const Dims& d);
int pipe_max_team();
const void* pipe_backward_kernel(const Dims& d, int variant, int* nt, int* k);

hipError_t read_expired_waits(void* header, hipStream_t st, int32_t* expired) {
    static_assert(sizeof(TeamHeader) <= kHeaderBytes, "the workspace header outgrew its place");
    TeamHeader h;
    hipError_t e = hipMemcpyAsync(&h, header, sizeof(TeamHeader), hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return e;
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return e;
    *expired = 0;
    if ((h.state & kHeaderMask) != kHeaderMagic || h.expired == 0u) return hipSuccess;
    *expired = h.expired > 0x7fffffffu ? 0x7fffffff : int32_t(h.expired);
    e = hipMemsetAsync(&static_cast<TeamHeader*>(header)->expired, 0, sizeof(unsigned int), st);
    if (e != hipSuccess) return e;
    return hipStreamSynchronize(st);
}

// Plans and launches one fused pass over channels [c0, c0 + cg).  Returns hipErrorNotSupported
// when the channel does not fit on chip (the caller then takes the streaming kernels).
hipError_t launch_fused(const Dims& d, const IndexParams& ip, bool backward, const FusedIo& io, float eps,
                        float momentum, void* header, void* slots, size_t slot_bytes, int c0, int cg, hipStream_t st,
                        const FusedMix* mix, bool order_streams) {
    // One read of each option per call: a concurrent bns_set_option cannot change a choice half way through.
    const int opt_variant = g_tuning.fused_variant, opt_keep_x = g_tuning.fused_keep_x, opt_pipe = g_tuning.fused_pipe;
    const int opt_team = g_tuning.fused_team, opt_path = g_tuning.path, opt_coop = g_tuning.fused_coop;
    const int opt_masked = g_tuning.fused_patch_mask;
    int devid = 0;
    hipError_t e = hipGetDevice(&devid);
    if (e != hipSuccess) return e;
    if (devid < 0 || devid >= 16) return hipErrorNotSupported;
    std::lock_guard<std::mutex> lock(g_dev_mutex);      // planning only; released before the launch returns
    DeviceInfo& di = g_dev[devid];
    if (di.cus == 0) {
        int cus = 0, coop = 0;
        if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, devid)) != hipSuccess) return e;
        if ((e = hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, devid)) != hipSuccess) return e;
        di.coop = coop;
        di.cus = cus;
    }
    if (!di.coop || di.cus <= 0) return hipErrorNotSupported;

    const uint32_t hwv = uint32_t(d.HW / d.vec);
    const uint32_t tot = uint32_t(d.N) * hwv;
    const int combo = combo_index(d);
    int kind = (backward ? 1 : (ip.shared.h_cnt * ip.shared.w_cnt == d.HW ? 0 : 2)) | (mix ? 4 : 0);

    // Choice of variant and team size, from sweeps on MI355X (64x256x56x56 fp32/bf16, 128x64x32x32,
    // 130x128x28x28):
    //  * a team of T blocks needs T * nt * kmax >= vectors per channel; T is then widened so that
    //    every block has work, and nudged (up to 2x) to the T that minimises rounds x vectors per
    //    thread, i.e. that leaves no half-empty last round;
    //  * candidate A = fewest rounds, then no exchange (T = 1), then the smallest variant;
    //  * backward, and forward with S = everything: (512 threads, 16 vectors), two blocks per
    //    compute unit, beats the bigger variants even when it needs more rounds (two teams per
    //    unit overlap one team's exchange and stores with the other's loads), so A is capped there;
    //  * forward with a sampled S saves only r of the bytes; it wins when all channels are in
    //    flight at once (one round), else the streaming kernels are faster.
    struct Plan {
        int v = -1, T = 0, blocks = 0;
        long rounds = 0;
    };
    auto plan_for = [&](int v, Plan* out) -> hipError_t {
        const Variant& va = kVariants[v];
        out->v = -1;
        int& bpc = di.blocks_per_cu[kind][combo][v];
        if (bpc == 0 && kernel_for(d, kind, v) == nullptr) bpc = -1;        // flavour not built for this variant
        if (bpc == 0) {
            int nb = 0;
            const hipError_t oe = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel_for(d, kind, v), va.nt, 0);
            if (oe != hipSuccess) return oe;
            bpc = nb > 0 ? nb : -1;
        }
        out->v = -1;
        if (bpc < 0) return hipSuccess;
        const long blocks = long(di.cus) * bpc;
        const long chunks = long((tot + va.nt - 1) / va.nt);                // nt-vector chunks per channel
        const long Tmin = (chunks + va.kmax - 1) / va.kmax;                 // members needed for one channel
        if (Tmin > blocks || Tmin > kMaxTeam) return hipSuccess;
        long bestT = 0, best_cost = 0, best_rounds = 0;
        // widen only while every thread still keeps >= 4 vectors: below that the exchange costs more
        // than the extra blocks bring
        long Thi = 2 * Tmin;
        if (long(cg) * Tmin < blocks) {
            Thi = blocks / cg;
            if (Thi > chunks / 4) Thi = chunks / 4;
            if (Thi < Tmin) Thi = Tmin;
        }
        for (long T = Tmin; T <= Thi && T <= kMaxTeam && T <= blocks; ++T) {
            const long teams = blocks / T < cg ? blocks / T : cg;
            const long rounds = (cg + teams - 1) / teams;
            const long cost = rounds * ((chunks + T - 1) / T + 2);          // +2: exchange and ramp per round
            if (bestT == 0 || cost < best_cost) {
                bestT = T;
                best_cost = cost;
                best_rounds = rounds;
            }
        }
        out->v = v;
        out->T = int(bestT);
        out->blocks = int(blocks);
        out->rounds = best_rounds;
        return hipSuccess;
    };
    // candidate A among the variants 0 .. last of the current kernel kind
    auto candidate = [&](int last, Plan* out) -> hipError_t {
        long best_key = -1;
        out->v = -1;
        for (int v = 0; v <= last; ++v) {
            Plan p;
            const hipError_t pe = plan_for(v, &p);
            if (pe != hipSuccess) return pe;
            if (p.v < 0) continue;
            const long key = p.rounds * 100000 + (p.T == 1 ? 0 : p.T <= 64 ? 1 : p.T) * 8 + v;
            if (out->v < 0 || key < best_key) {
                *out = p;
                best_key = key;
            }
        }
        return hipSuccess;
    };
    Plan chosen;
    if (opt_variant > 0) {
        if (backward && opt_keep_x == 1) {        // both forced: the keep-x flavour of that variant, if built
            kind |= 2;
            if ((e = plan_for(opt_variant - 1, &chosen)) != hipSuccess) return e;
            if (chosen.v < 0) kind &= ~2;
        }
        if (chosen.v < 0 && (e = plan_for(opt_variant - 1, &chosen)) != hipSuccess) return e;
    } else {
        if ((e = candidate(kNumVariants - 1, &chosen)) != hipSuccess) return e;
        const bns_box& sb = ip.shared;
        const bool everything = !ip.per_channel && sb.n_cnt == d.N && sb.h_cnt == d.H && sb.w_cnt == d.W;
        const bool patch = sb.h_cnt * sb.w_cnt != d.HW;
        constexpr int kTwoPerUnit = 4;                                       // {512, 16}
        // (not when the big variant holds a channel per block: without any exchange it is the faster one, full BN
        // forward at 64x256x56x56 bf16 41 against 47 us)
        if (chosen.v > kTwoPerUnit && (backward || (everything && chosen.T > 1))) {
            Plan p;
            if ((e = plan_for(kTwoPerUnit, &p)) != hipSuccess) return e;
            if (p.v >= 0) chosen = p;
        }
        // (Eq. 4 has no such alternative: its streaming forward is four launches)
        if (chosen.v >= 0 && !backward && !everything && chosen.rounds > 1 && opt_path != 2 && !mix)
            return hipErrorNotSupported;
        // Backward needs x a second time on S.  When that is most of the channel (full BN), or a patch of
        // every plane (the second read then fetches scattered pieces of lines), both tensors stay on chip:
        // up to (512 threads, 8 + 8 vectors), the register cost of (512, 16).  Measured at 64x256x56x56 fp32:
        // full BN 153 -> 130 us, Feature Sampling 134 -> 127; 128x64x32x32 Feature Sampling 30 -> 22.
        // Whole planes of a few samples (Batch Sampling, VDN) re-read little and lose more to the larger teams;
        // Eq. 4 reads two sets again and gains (130x128x28x28, 2 virtual + 4 of 128 real samples: 39 -> 36 us).
        constexpr int kKeepXLast = 3;                                        // {512, 8}
        const bool keep_x = opt_keep_x == 1 || (opt_keep_x == 0 && (everything || patch || mix));
        if (backward && keep_x) {
            kind |= 2;
            Plan p;
            if ((e = candidate(kKeepXLast, &p)) != hipSuccess) return e;
            if (p.v >= 0)
                chosen = p;
            else
                kind &= ~2;
        }
    }
    // Backward over several rounds: the pipelined kernel (bns_fused_pipe.hip), which holds the dy vectors of two
    // channels per member so that loads stay in flight across the exchange, and parks x in LDS so that no mode
    // reads anything twice.  "fused_pipe": 0 = whenever it applies, 1..n = that variant, 16 = never.  (A forward
    // kernel built the same way was 10 us slower than the plain one at 64x256x56x56 and was dropped: with one
    // tensor to read there is no second stream of loads to put between the prefetch and the stores.)
    const void* pipe_kernel = nullptr;
    int pipe_nt = 0, pipe_k = 0;
    const bool pipe_forced = opt_pipe > 0 && opt_pipe <= pipe_variant_count();
    const bool pipe_auto = opt_pipe == 0 && opt_variant == 0 && opt_keep_x == 0;
    // (its per-vector byte offsets are 32-bit: tensors below 4 GiB)
    const bool pipe_fits = uint64_t(d.N) * uint64_t(d.C) * uint64_t(d.HW) * (d.dtype == BNS_F32 ? 4u : 2u) < (uint64_t(1) << 32);
    if (backward && !mix && pipe_fits && (pipe_forced || pipe_auto)) {
        struct PipePlan {
            const void* kernel = nullptr;
            int nt = 0, k = 0;
            long T = 0, rounds = 0, blocks = 0;
            double cost = 0.0;
        };
        auto pipe_plan = [&](int pv, PipePlan* out) -> hipError_t {
            out->kernel = nullptr;
            int nt = 0, k = 0;
            const void* kp = pipe_backward_kernel(d, pv, &nt, &k);
            if (!kp) return hipSuccess;
            int& bpc = di.pipe_blocks_per_cu[combo][pv];
            if (bpc == 0) {
                int nb = 0;
                const hipError_t oe = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kp, nt, 0);
                if (oe != hipSuccess) return oe;
                bpc = nb > 0 ? nb : -1;
            }
            if (bpc < 0) return hipSuccess;
            const long blocks = long(di.cus) * bpc;
            const long chunks = long((tot + nt - 1) / nt);
            const long Tmin = (chunks + k - 1) / k;
            const long Tmax = blocks < pipe_max_team() ? blocks : pipe_max_team();
            long bestT = 0, best_rounds = 0;
            double best_cost = 0.0;
            for (long T = Tmin; T <= 2 * Tmin && T <= Tmax; ++T) {
                const long teams = blocks / T < cg ? blocks / T : cg;
                const long rounds = (cg + teams - 1) / teams;
                // a round lasts as long as its busiest member's share (whole chunks) plus the exchange, whose wait and
                // sum grow with the team (128 per member: between the two shapes it was fitted to -- 64x256x56x56,
                // teams of 16 x 448 threads, 1 us faster than 14 x 512; 64x64x112x112, 56 x 512 5 us faster than 64 x 448)
                const double cost = double(rounds) * ((double((chunks + T - 1) / T) + 2.0) * double(nt) + 128.0 * double(T));
                if (bestT == 0 || cost < best_cost) {
                    bestT = T;
                    best_cost = cost;
                    best_rounds = rounds;
                }
            }
            if (opt_team > 0 && opt_team >= Tmin && opt_team <= Tmax)
                bestT = opt_team;
            if (bestT == 0) return hipSuccess;
            out->kernel = kp;
            out->nt = nt;
            out->k = k;
            out->T = bestT;
            out->rounds = best_rounds;
            out->blocks = blocks;
            out->cost = best_cost;
            return hipSuccess;
        };
        PipePlan pp;
        if (pipe_forced) {
            if ((e = pipe_plan(opt_pipe - 1, &pp)) != hipSuccess) return e;
        } else {
            // 512 or 448 threads, whichever cuts the channel into shares with less padding.  Measured at
            // 64x256x56x56 (fp32, 8 rounds): 115-117 us for every mode against 127-130 for the plain kernels; bf16
            // (6 rounds) 63-64 against 66 (Batch Sampling) and 71 (full BN).  With two rounds (128x64x32x32,
            // 130x128x28x28) the plain kernels are faster, and so they are for a patch of every plane in bf16 whose
            // rows are not a whole number of vectors: most vectors of 8 elements then need the test of row and
            // column element by element (70 against 68 us).  With whole vectors per row the patch is a run of
            // columns in each vector: 71 us against 73-74 for the plain kernel that keeps x in registers.
            const bns_box& sb = ip.shared;
            const bool patch_bf16 = d.vec == 8 && d.W % d.vec != 0 && (ip.per_channel || sb.w_cnt != d.W || sb.w0 != 0);
            PipePlan alt;
            if ((e = pipe_plan(pipe_default_variant(d), &pp)) != hipSuccess) return e;
            if (pipe_alternative_variant(d) >= 0) {
                if ((e = pipe_plan(pipe_alternative_variant(d), &alt)) != hipSuccess) return e;
                if (alt.kernel && (!pp.kernel || alt.cost < pp.cost)) pp = alt;
            }
            if (pp.kernel && (pp.rounds < 3 || patch_bf16)) pp.kernel = nullptr;
        }
        if (pp.kernel) {
            pipe_kernel = pp.kernel;
            pipe_nt = pp.nt;
            pipe_k = pp.k;
            kind = 1;
            chosen.v = 0;
            chosen.T = int(pp.T);
            chosen.blocks = int(pp.blocks);
        }
    }
    if (chosen.v < 0) return hipErrorNotSupported;
    const int best = chosen.v, bestT = chosen.T, best_blocks = chosen.blocks;
    const int launch_nt = pipe_kernel ? pipe_nt : kVariants[best].nt;
    const int launch_k = pipe_kernel ? pipe_k : kVariants[best].kmax;

    FusedArgs A;
    A.x = io.x;
    A.dy = io.dy;
    A.out = io.out;
    A.gamma = io.gamma;
    A.beta = io.beta;
    A.save_mean = io.save_mean;
    A.save_invstd = io.save_invstd;
    A.running_mean = io.running_mean;
    A.running_var = io.running_var;
    A.dgamma = io.dgamma;
    A.dbeta = io.dbeta;
    A.hdr = static_cast<TeamHeader*>(header);
    A.slots = static_cast<unsigned long long*>(slots);
    A.ip = ip;
    A.hwv_div = make_fastdiv(hwv);
    A.w_div = make_fastdiv(uint32_t(d.W));
    A.wv_div = make_fastdiv(uint32_t(d.W / d.vec > 0 ? d.W / d.vec : 1));       // used when W is a multiple of vec
    A.patch_stage = 0;
    A.rows_whole = d.W % d.vec == 0;
    A.chw_div = make_fastdiv(uint32_t(d.C) * uint32_t(d.HW));       // C * HW < 2^31 (limits of bns_shape)
    A.C = d.C;
    A.W = d.W;
    A.HW = d.HW;
    A.c0 = c0;
    A.cg = cg;
    A.T = bestT;
    A.num_teams = best_blocks / bestT;
    if (A.num_teams > cg) A.num_teams = cg;
    A.tot = tot;
    const uint32_t rounds = uint32_t((cg + A.num_teams - 1) / A.num_teams);
    A.stamp_advance = (mix ? 2u : 1u) * rounds + 1u;               // Eq. 4 forward exchanges twice per round
    A.stamp_seed = g_stamp.fetch_add(1u);
    const int spin = g_tuning.test_spin_limit;
    A.spin_limit = spin > 0 ? uint32_t(spin) : kSpinLimit;
    A.mute = g_tuning.test_mute_exchange;
    A.eps = eps;
    A.momentum = momentum;
    const bns_box& b = ip.shared;
    A.s = double(b.n_cnt) * double(b.h_cnt) * double(b.w_cnt);
    A.s_cnt = uint32_t(b.n_cnt) * uint32_t(b.h_cnt) * uint32_t(b.w_cnt);
    A.n_v = 0;
    A.mix_beta = A.w_v = A.w_s = 0.f;
    A.s_v = 1.0;
    A.mean_parts = nullptr;
    if (mix) {
        A.n_v = mix->n_v;
        A.mix_beta = mix->mix_beta;
        A.s_v = double(mix->n_v) * double(d.HW);
        A.w_v = float(double(mix->mix_beta) / A.s_v);
        A.w_s = float((1.0 - double(mix->mix_beta)) / A.s);
        A.mean_parts = mix->mean_parts;
    }
    A.patch_div = make_fastdiv(uint32_t(b.h_cnt) * uint32_t(b.w_cnt));
    A.pw_div = make_fastdiv(uint32_t(b.w_cnt));
    A.inv_s = float(1.0 / A.s);

    const int grid = A.num_teams * bestT;
    if (size_t(grid) * 2 * 2 * sizeof(unsigned long long) > slot_bytes) return hipErrorNotSupported;
    {
        const uint64_t chunks = (uint64_t(tot) + launch_nt - 1) / launch_nt;
        if ((chunks + bestT - 1) / bestT > uint64_t(launch_k)) return hipErrorNotSupported;
    }
    const void* kernel = pipe_kernel ? pipe_kernel : kernel_for(d, kind, best);
    // A patch, and the block holds its channel alone: nothing happens while the vectors arrive that separately
    // read patch elements could run ahead for, so the statistics come from the registers
    // (64x256x56x56 bf16, 14x14 patch: forward 49.4 -> 42.8 us; full BN on the same tensor 41.5).
    if (kind == 2 && !pipe_kernel && best >= kMaskedFirstVariant && (opt_masked == 1 || (opt_masked == 0 && bestT == 1))) {
        const void* masked = masked_forward_kernel(d, best);
        if (masked) {
            kernel = masked;
            // one block per channel, and the vectors that touch the patch (the widest span a patch of w_cnt columns
            // can have, whatever its first column) fit the kernel's staging array
            const uint64_t span = uint64_t(d.vec - 1 + ip.shared.w_cnt - 1) / uint64_t(d.vec) + 1u;
            const uint64_t slots = uint64_t(ip.shared.n_cnt) * uint64_t(ip.shared.h_cnt) * span;
            A.patch_stage = (bestT == 1 && slots <= uint64_t(kStageSlots)) ? 1 : 0;
        }
    }
    if (!backward) t_last_fused_forward = kernel == kernel_for(d, kind, best) ? 1 : 2;
    void* params[] = {&A};

    // Kernels whose blocks wait for each other must not share the device with one another: two of them, each with
    // part of its grid resident, would wait for blocks that the other keeps out.  Within a process they are therefore
    // chained across streams: when such a launch goes to another stream than the one before it, an event is
    // recorded on that earlier stream (behind the earlier launch) and the new stream waits for it.  A caller that
    // stays on one stream pays nothing.  Not while a stream is being captured (the event would belong to the
    // graph); a graph that holds such launches must not run beside other calls.
    bool chain = false;
    if (bestT > 1 && order_streams) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        chain = hipStreamIsCapturing(st, &cap) == hipSuccess && cap == hipStreamCaptureStatusNone;
        (void)hipGetLastError();
    }
    if (chain && di.chain_active && di.chain_stream != st) {
        if (!di.chain_event && hipEventCreateWithFlags(&di.chain_event, hipEventDisableTiming) != hipSuccess)
            di.chain_event = nullptr;
        // (an earlier stream that has been destroyed meanwhile refuses the record: nothing is left to wait for)
        if (di.chain_event && hipEventRecord(di.chain_event, di.chain_stream) == hipSuccess &&
            (e = hipStreamWaitEvent(st, di.chain_event, 0)) != hipSuccess)
            return e;
        (void)hipGetLastError();
    }
    g_launch_count.fetch_add(1, std::memory_order_relaxed);
    if (backward) t_last_fused_backward = pipe_kernel ? 3 : (kind & 2) ? 2 : 1;
    e = opt_coop ? hipLaunchCooperativeKernel(kernel, dim3(grid), dim3(launch_nt), params, 0, st)
                            : hipLaunchKernel(kernel, dim3(grid), dim3(launch_nt), params, 0, st);
    if (e == hipSuccess && chain) {
        di.chain_active = true;
        di.chain_stream = st;
    }
    return e;
}

}  // namespace bns
