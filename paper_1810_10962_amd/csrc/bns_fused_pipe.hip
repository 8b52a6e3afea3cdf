// Single-launch backward pass, software-pipelined over the channels a team owns.
//
// The kernels of bns_fused.hip take one channel at a time: load dy and x, add up, exchange the sums with the
// team, write dx, and only then touch the next channel.  Between a member's last load and its first store lie
// its block reduction and the exchange with its team-mates, a few microseconds in which it has nothing in
// flight; with every block of the device in step, HBM idles for that part of each round.  Here a member holds
// the dy vectors of TWO channels (K vectors each): the loads of channel k+1 are issued after the member has
// published its sums of channel k and before it waits for the team's, so that they, and then the stores of
// channel k, keep memory busy across the exchange.  Same teams, slots, stamps and summation order as the
// kernels of bns_fused.hip; results are bit-identical to theirs for the same (block size, team size).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "bns_device.hpp"
#include "bns_fused_device.hpp"
#include "bns_internal.hpp"

namespace bns {

namespace {

constexpr int kPipeMaxTeam = 128;   // members of a team of the pipelined kernel (its exchange buffer is sized for this)

// Sum over the 64 lanes of a wave, returned as a wave-uniform value.  Inclusive scan with data-parallel-primitive
// moves (shifts of 1, 2, 4, 8 lanes inside each row of 16, then the last lane of row 0 / row 2 broadcast into the
// next row, then lane 31 into the upper half), after which lane 63 holds the total.  Unlike a butterfly of
// cross-lane shuffles this needs no lane-index registers, which matter in a kernel that lives on its register
// budget; the order of the additions is fixed, so results are reproducible.
__device__ __forceinline__ float wave_total(float v) {
    auto shifted = [](float x, auto ctrl, auto row_mask) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value,
                                                                    decltype(row_mask)::value, 0xf, true));
    };
    using std::integral_constant;
    v += shifted(v, integral_constant<int, 0x111>{}, integral_constant<int, 0xf>{});   // row_shr:1
    v += shifted(v, integral_constant<int, 0x112>{}, integral_constant<int, 0xf>{});   // row_shr:2
    v += shifted(v, integral_constant<int, 0x114>{}, integral_constant<int, 0xf>{});   // row_shr:4
    v += shifted(v, integral_constant<int, 0x118>{}, integral_constant<int, 0xf>{});   // row_shr:8
    v += shifted(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{});   // row_bcast:15 into rows 1, 3
    v += shifted(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{});   // row_bcast:31 into rows 2, 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// Block-wide sum of (a, b) over NT threads, returned to every thread: one value per wave through LDS, added in
// wave order by every thread.
template <int NT>
__device__ __forceinline__ void block_total2(float& a, float& b, float* red) {
    a = wave_total(a);
    b = wave_total(b);
    constexpr int nw = NT / kWave;
    if (nw > 1) {
        const int wave = threadIdx.x / kWave;
        __syncthreads();                       // red[] may still be read from the previous use
        if (threadIdx.x % kWave == 0) {
            red[wave] = a;
            red[nw + wave] = b;
        }
        __syncthreads();
        float sa = red[0], sb = red[nw];
#pragma unroll
        for (int w = 1; w < nw; ++w) {
            sa += red[w];
            sb += red[nw + w];
        }
        a = sa;
        b = sb;
    }
}

// Waits for the pair of every member of the team (thread t polls member t's slot) and returns the totals, added
// in member order in fp64 by every thread (so all members, and all threads, get the same bits).
template <int NT>
__device__ __forceinline__ void team_totals(const FusedArgs& A, uint32_t stamp0, int team_first_block, uint32_t it, float a,
                                            float b, double& ta, double& tb, float* team_lds) {
    if (A.T == 1) {
        ta = double(a);
        tb = double(b);
        return;
    }
    const uint32_t stamp = stamp0 + it;
    unsigned long long* base = A.slots + size_t(it & 1u) * gridDim.x * 2;
    for (int t = threadIdx.x; t < A.T; t += NT) {
        float pa, pb;
        poll_pair(A, base + size_t(team_first_block + t) * 2, stamp, pa, pb);      // NaN if the wait ran out
        team_lds[2 * t] = pa;
        team_lds[2 * t + 1] = pb;
    }
    __syncthreads();
    double sa = 0.0, sb = 0.0;
#pragma unroll 1
    for (int t = 0; t < A.T; ++t) {
        sa += double(team_lds[2 * t]);
        sb += double(team_lds[2 * t + 1]);
    }
    ta = sa;
    tb = sb;
    __syncthreads();                           // team_lds is written again by the next channel's wait
}

// LDS vector of 16 bytes (8 bytes for 4-wide bf16), one per thread and x vector.
template <typename R>
struct alignas(sizeof(R)) Parked {
    R r;
};

// What a thread knows about its K vectors of a channel.  The position of vector k inside a channel (sample, place in
// the plane) is the same for every channel the team takes, so byte offsets, validity and membership in S are worked out
// once per launch, and a round spends no arithmetic on addresses: a load is "channel base (scalar) + 32-bit offset".
// (Tensors of 4 GiB and more take the kernels of bns_fused.hip.)
//   cls, two bits per vector: 0 = no element in S, 1 = every element in S, 2 = some (a patch row crosses it, or
//   the patch location depends on the channel): membership is then tested element by element
//   valid, one bit per vector: it exists (vectors past the end of the channel are mapped onto its last vector so that
//   every load is unconditional; they are weighted 0 in the sums and never stored)
template <typename T, int V, int K, int NT>
struct BackwardPipe {
    typedef RawVec<T, V> RV;
    typedef typename RV::raw_t raw_t;
    static constexpr int XB = V == 8 ? 2 : K < 3 ? K : (NT == 448 || K < 4) ? 3 : 4;      // x vectors in flight per thread (registers decide)

    const FusedArgs& A;
    uint32_t off[K];       // byte offset of vector k from the channel's first element
    uint32_t cls, valid;

    __device__ __forceinline__ BackwardPipe(const FusedArgs& a, int j) : A(a) {
        // member j owns the NT-vector chunks j, j + T, j + 2T, ... of the channel
        const uint32_t first = uint32_t(j) * NT + threadIdx.x, step = uint32_t(a.T) * NT;
        const uint32_t hwv = a.hwv_div.d;
        const bns_box& b = a.ip.shared;
        const bool full_rows = b.w0 == 0 && b.w_cnt == a.W;
        cls = valid = 0;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            uint32_t i = first + uint32_t(k) * step;
            const bool ok = i < a.tot;
            i = i < a.tot ? i : a.tot - 1u;
            const uint32_t n = fdiv(i, a.hwv_div);
            const uint32_t e0 = (i - n * hwv) * V;
            off[k] = (n * uint32_t(a.C) * uint32_t(a.HW) + e0) * uint32_t(sizeof(T));     // < 2^32: checked by the host
            valid |= uint32_t(ok) << k;
            const uint32_t lo = uint32_t(b.h0) * a.W, hi = uint32_t(b.h0 + b.h_cnt) * a.W;
            const bool touches = n >= uint32_t(b.n0) && n < uint32_t(b.n0 + b.n_cnt) && e0 + V > lo && e0 < hi;
            const bool inside = full_rows && touches && e0 >= lo && e0 + V <= hi;
            const uint32_t c = a.ip.per_channel ? 2u : inside ? 1u : touches ? 2u : 0u;
            cls |= c << (2 * k);
        }
    }

    template <typename P>
    static __device__ __forceinline__ P* at(P* base, uint32_t byte_off) {
        // pointer arithmetic, not integer arithmetic: the access stays a global one (an address rebuilt from an integer
        // is a flat address, whose loads also count as LDS traffic and stall every wait for the LDS)
        typedef std::conditional_t<std::is_const<P>::value, const char, char> byte_t;
        return reinterpret_cast<P*>(reinterpret_cast<byte_t*>(base) + byte_off);
    }

    // Issues the loads of channel c that can run ahead: all K dy vectors and the first XB x vectors.
    __device__ __forceinline__ void prefetch(raw_t (&g)[K], raw_t (&x0)[XB], int c) const {
        const T* gc = static_cast<const T*>(A.dy) + size_t(c) * A.HW;
        const T* xc = static_cast<const T*>(A.x) + size_t(c) * A.HW;
#pragma unroll
        for (int k = 0; k < K; ++k) g[k] = RV::ld(at(gc, off[k]));
#pragma unroll
        for (int u = 0; u < XB; ++u) x0[u] = RV::ld(at(xc, off[u]));
    }

    // Sums of Eq. 5 over this thread's share of channel c.  x is streamed XB vectors at a time (the first batch
    // is already on its way) and parked in LDS for the dx pass, so that no byte is read twice.
    __device__ __forceinline__ void sums(raw_t (&g)[K], raw_t (&x0)[XB], int c, float mu, Parked<raw_t>* park, float& s1,
                                         float& s2) const {
        const T* xc = static_cast<const T*>(A.x) + size_t(c) * A.HW;
#pragma unroll
        for (int k0 = 0; k0 < K; k0 += XB) {
            raw_t xv[XB];
#pragma unroll
            for (int u = 0; u < XB; ++u) {
                if (k0 == 0)
                    xv[u] = x0[u];
                else if (k0 + u < K)
                    xv[u] = RV::ld(at(xc, off[k0 + u]));
            }
#pragma unroll
            for (int u = 0; u < XB; ++u) {
                if (k0 + u < K) {
                    const int k = k0 + u;
                    float fg[V], fx[V];
                    RV::unpack(g[k], fg);
                    RV::unpack(xv[u], fx);
                    park[k * NT + threadIdx.x].r = xv[u];
                    float t1 = fg[0], t2 = fg[0] * (fx[0] - mu);            // the vector's own sums first,
#pragma unroll
                    for (int e = 1; e < V; ++e) {
                        t1 += fg[e];
                        t2 = fmaf(fg[e], fx[e] - mu, t2);
                    }
                    const float m = ((valid >> k) & 1u) ? 1.f : 0.f;      // then weighted 1 or 0
                    s1 = fmaf(m, t1, s1);
                    s2 = fmaf(m, t2, s2);
                }
            }
        }
    }

    // Eq. 6 over this thread's share of channel c; x comes back from LDS (each thread reads what it parked itself)
    __device__ __forceinline__ void write_dx(raw_t (&g)[K], int c, const bns_box& b, float a, float k1, float k2,
                                             float mu, const Parked<raw_t>* park) const {
        T* dc = static_cast<T*>(A.out) + size_t(c) * A.HW;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if ((valid >> k) & 1u) {
                float f[V];
                RV::unpack(g[k], f);
                const uint32_t ck = (cls >> (2 * k)) & 3u;
                if (ck == 0u) {
#pragma unroll
                    for (int e = 0; e < V; ++e) f[e] *= a;
                } else {
                    float fx[V];
                    RV::unpack(park[k * NT + threadIdx.x].r, fx);
                    if (ck == 1u) {
#pragma unroll
                        for (int e = 0; e < V; ++e) f[e] = fmaf(a, f[e], -fmaf(k2, fx[e] - mu, k1));
                    } else {
                        // position of the vector from its offset: sample, then row and column of its first element
                        // (worked out here, from an opaque copy, every time: hoisted out of the channel loop these
                        // few values per vector would cost more registers than the kernel has)
                        const uint32_t el = opaque(off[k]) / uint32_t(sizeof(T));
                        const uint32_t n = fdiv(el, A.chw_div);
                        const uint32_t e0 = el - n * A.chw_div.d;
                        uint32_t h = fdiv(e0, A.w_div);
                        uint32_t w = e0 - h * uint32_t(A.W);
                        const bool n_in = n >= uint32_t(b.n0) && n < uint32_t(b.n0 + b.n_cnt);
                        if (A.rows_whole) {
                            // a row is a whole number of vectors: the vector lies in one row, and the elements of S
                            // in it are a run [lo, hi) of its columns
                            const bool row_in = n_in && h - uint32_t(b.h0) < uint32_t(b.h_cnt);
                            const int32_t lo = row_in ? max(b.w0 - int32_t(w), 0) : V;
                            const int32_t hi = min(b.w0 + b.w_cnt - int32_t(w), V);
#pragma unroll
                            for (int e = 0; e < V; ++e) {
                                const float corr = (e >= lo && e < hi) ? fmaf(k2, fx[e] - mu, k1) : 0.f;
                                f[e] = fmaf(a, f[e], -corr);
                            }
                        } else {
#pragma unroll
                            for (int e = 0; e < V; ++e) {
                                const float corr = (n_in && in_hw(b, h, w)) ? fmaf(k2, fx[e] - mu, k1) : 0.f;
                                f[e] = fmaf(a, f[e], -corr);
                                if (++w == uint32_t(A.W)) {
                                    w = 0;
                                    ++h;
                                }
                            }
                        }
                    }
                }
                RV::st(at(dc, off[k]), RV::pack(f));
            }
        }
    }
};

template <typename T, int V, int K, int NT>
__global__ __launch_bounds__(NT, 4) void fused_backward_pipe_kernel(FusedArgs A) {
    typedef BackwardPipe<T, V, K, NT> P;
    typedef typename P::raw_t raw_t;
    __shared__ Parked<raw_t> park[K * NT];
    __shared__ float red[2 * (NT / kWave)];
    __shared__ float team_lds[2 * kPipeMaxTeam];
    __shared__ uint32_t stamp_word[3];
    const int team = blockIdx.x / A.T;                     // the grid is exactly num_teams * T blocks
    const int j = blockIdx.x - team * A.T;
    const P p(A, j);

    raw_t ga[K], gb[K], x0[P::XB];

    // One channel: its dy is in `cur` and its first x vectors in x0 (loads issued earlier); `nxt` and x0 receive
    // the next channel's.
    auto one_channel = [&](raw_t(&cur)[K], raw_t(&nxt)[K], int cl, uint32_t it) {
        const int c = A.c0 + cl;
        const bns_box b = box_of_channel(A.ip, c);
        const float mu = settled(A.save_mean[c]);
        const float r = settled(A.save_invstd[c]);
        const float ga_c = settled(A.gamma[c]);
        float s1 = 0.f, s2 = 0.f;
        p.sums(cur, x0, c, mu, park, s1, s2);
        block_total2<NT>(s1, s2, red);
        const uint32_t stamp0 = read_stamp(A, stamp_word);    // drawn before the loop; the barriers above lie between
        team_publish(A, stamp0, team * A.T, j, it, s1, s2);
        if (cl + A.num_teams < A.cg) p.prefetch(nxt, x0, c + A.num_teams);     // in flight across the exchange
        double t1, t2;
        team_totals<NT>(A, stamp0, team * A.T, it, s1, s2, t1, t2, team_lds);
        const float dbeta = float(t1);
        const float dgamma = float(t2 * double(r));
        if (j == 0 && threadIdx.x == 0) {
            A.dbeta[c] = dbeta;
            A.dgamma[c] = dgamma;
        }
        const float a = ga_c * r;
        p.write_dx(cur, c, b, a, a * A.inv_s * dbeta, a * A.inv_s * dgamma * r, mu, park);
    };

    int cl = team;
    uint32_t it = 0;
    if (cl < A.cg) p.prefetch(ga, x0, A.c0 + cl);
    stamp_accept(A, stamp_request(A), stamp_word);             // (every block of the grid; the first loads are on their way)
    while (cl < A.cg) {
        one_channel(ga, gb, cl, it);
        cl += A.num_teams;
        ++it;
        if (cl >= A.cg) break;
        one_channel(gb, ga, cl, it);
        cl += A.num_teams;
        ++it;
    }
    team_done(A, j, read_stamp(A, stamp_word));
}

struct PipeVariant {
    int nt, k;
};
// (threads per block, vectors per thread and channel)
constexpr PipeVariant kPipeVariants[] = {{512, 4}, {512, 5}, {512, 7}, {448, 7}, {448, 4}, {256, 7}};
constexpr int kNumPipeVariants = sizeof(kPipeVariants) / sizeof(kPipeVariants[0]);

template <typename T, int V>
const void* pipe_ptr(int variant) {
    switch (variant) {
        case 0: return reinterpret_cast<const void*>(&fused_backward_pipe_kernel<T, V, 4, 512>);
        case 1: return reinterpret_cast<const void*>(&fused_backward_pipe_kernel<T, V, 5, 512>);
        case 2: return reinterpret_cast<const void*>(&fused_backward_pipe_kernel<T, V, 7, 512>);
        case 3: return reinterpret_cast<const void*>(&fused_backward_pipe_kernel<T, V, 7, 448>);
        case 4: return reinterpret_cast<const void*>(&fused_backward_pipe_kernel<T, V, 4, 448>);
        case 5: return reinterpret_cast<const void*>(&fused_backward_pipe_kernel<T, V, 7, 256>);
    }
    return nullptr;
}

}  // namespace

int pipe_variant_count() { return kNumPipeVariants; }
int pipe_max_team() { return kPipeMaxTeam; }
// Default variants.  (512 or 448 threads, 7 vectors per channel) uses about 120 registers, so two blocks share a
// compute unit; 8 bf16 per vector unpack into twice the registers, which leaves room for 4 vectors per channel
// (with more the compiler spills, and a spilling variant is half as fast).
int pipe_default_variant(const Dims& d) { return d.vec == 8 ? 0 : 2; }
int pipe_alternative_variant(const Dims& d) { return d.vec == 8 ? 4 : 3; }   // the same with 448 threads

// The pipelined backward kernel of variant `variant` for this storage type and access width (vector
// accesses only), with its block size and vectors per thread and channel; nullptr if there is none.
const void* pipe_backward_kernel(const Dims& d, int variant, int* nt, int* k) {
    if (variant < 0 || variant >= kNumPipeVariants || d.vec == 1) return nullptr;
    *nt = kPipeVariants[variant].nt;
    *k = kPipeVariants[variant].k;
    if (d.dtype == BNS_F32) return pipe_ptr<float, 4>(variant);
    return d.vec == 8 ? pipe_ptr<bf16_t, 8>(variant) : pipe_ptr<bf16_t, 4>(variant);
}

}  // namespace bns
