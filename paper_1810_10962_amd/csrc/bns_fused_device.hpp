// Device-side pieces shared by the single-launch ("fused") kernels: packed register vectors, the kernel
// argument block, and the exchange of partial sums between the blocks of a team.
#pragma once
#include <hip/hip_runtime.h>

#include "bns_device.hpp"
#include "bns_internal.hpp"

namespace bns {
namespace {

// ---------------------------------------------------------------------------------------
// RawVec<T, V>: V storage elements as they sit in memory (kept packed in registers).
// ---------------------------------------------------------------------------------------
template <typename T, int V>
struct RawVec;

template <>
struct RawVec<float, 1> {
    typedef float raw_t;
    static __device__ __forceinline__ raw_t ld(const float* p) { return __builtin_nontemporal_load(p); }
    static __device__ __forceinline__ void st(float* p, raw_t r) { __builtin_nontemporal_store(r, p); }
    static __device__ __forceinline__ void unpack(raw_t r, float* f) { f[0] = r; }
    static __device__ __forceinline__ raw_t pack(const float* f) { return f[0]; }
};
template <>
struct RawVec<float, 4> {
    typedef float raw_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ raw_t ld(const float* p) {
        return __builtin_nontemporal_load(reinterpret_cast<const raw_t*>(p));
    }
    static __device__ __forceinline__ void st(float* p, raw_t r) {
        __builtin_nontemporal_store(r, reinterpret_cast<raw_t*>(p));
    }
    static __device__ __forceinline__ void unpack(raw_t r, float* f) {
        f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
    }
    static __device__ __forceinline__ raw_t pack(const float* f) { return raw_t{f[0], f[1], f[2], f[3]}; }
};
template <>
struct RawVec<bf16_t, 1> {
    typedef uint16_t raw_t;
    static __device__ __forceinline__ raw_t ld(const bf16_t* p) { return p->bits; }
    static __device__ __forceinline__ void st(bf16_t* p, raw_t r) { p->bits = r; }
    static __device__ __forceinline__ void unpack(raw_t r, float* f) { f[0] = bf16_to_f32(r); }
    static __device__ __forceinline__ raw_t pack(const float* f) { return uint16_t(f32_to_bf16(f[0])); }
};
template <>
struct RawVec<bf16_t, 4> {
    typedef uint32_t raw_t __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ raw_t ld(const bf16_t* p) {
        return __builtin_nontemporal_load(reinterpret_cast<const raw_t*>(p));
    }
    static __device__ __forceinline__ void st(bf16_t* p, raw_t r) {
        __builtin_nontemporal_store(r, reinterpret_cast<raw_t*>(p));
    }
    static __device__ __forceinline__ void unpack(raw_t r, float* f) {
        f[0] = bf16_to_f32(r.x & 0xFFFFu); f[1] = __uint_as_float(r.x & 0xFFFF0000u);
        f[2] = bf16_to_f32(r.y & 0xFFFFu); f[3] = __uint_as_float(r.y & 0xFFFF0000u);
    }
    static __device__ __forceinline__ raw_t pack(const float* f) {
        return raw_t{pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3])};
    }
};
template <>
struct RawVec<bf16_t, 8> {
    typedef uint32_t raw_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ raw_t ld(const bf16_t* p) {
        return __builtin_nontemporal_load(reinterpret_cast<const raw_t*>(p));
    }
    static __device__ __forceinline__ void st(bf16_t* p, raw_t r) {
        __builtin_nontemporal_store(r, reinterpret_cast<raw_t*>(p));
    }
    static __device__ __forceinline__ void unpack(raw_t r, float* f) {
        f[0] = bf16_to_f32(r.x & 0xFFFFu); f[1] = __uint_as_float(r.x & 0xFFFF0000u);
        f[2] = bf16_to_f32(r.y & 0xFFFFu); f[3] = __uint_as_float(r.y & 0xFFFF0000u);
        f[4] = bf16_to_f32(r.z & 0xFFFFu); f[5] = __uint_as_float(r.z & 0xFFFF0000u);
        f[6] = bf16_to_f32(r.w & 0xFFFFu); f[7] = __uint_as_float(r.w & 0xFFFF0000u);
    }
    static __device__ __forceinline__ raw_t pack(const float* f) {
        return raw_t{pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                     pack_bf16x2(f[6], f[7])};
    }
};

constexpr int kMaxTeam = 1024;            // members of a team (T)
constexpr uint32_t kSpinLimit = 1u << 21; // polls before a missing team-mate is given up on (default)

// First bytes of a workspace that the single-launch kernels have used.  Exchange stamps must never repeat in a
// workspace, under HIP graph replay either, so they are counted on the device.  `state` = {magic, first stamp of the
// next launch}: every block reads it on entry (a plain load: hundreds of blocks adding to one counter at once would
// cost them microseconds each).  Member 0 of every team adds one to `done` when the team has finished its last
// channel -- by then every member has taken part in every exchange, so it has read the header -- and the one that
// completes the count puts the following launch's stamp and a zero count in place.  (Launches that share a workspace
// are ordered on one stream.)  A workspace need not be initialised by the caller: the first block that finds no
// magic sets the words up, the others wait for it; chance bytes that look like the magic are as good a start as any.
// `expired` counts waits for a team-mate that ran out.
// A per-channel constant that came straight from a load and is used inside the (divergent) blocks of the unrolled
// store loops: the compiler's wait-count bookkeeping loses track of such a register at the joins and waits for
// "everything outstanding" before each use -- which includes the stores of the previous block, so the stores of a
// thread would go out one at a time.  Passing the value through an empty asm ends its life as a load result.
// (The stores of a thread now leave back to back: 0.6 us of 18 in the forward kernel at 128x64x32x32; at 64x256x56x56,
// where many blocks share a unit, the launch times did not change measurably.)
__device__ __forceinline__ float settled(float v) {
    asm volatile("" : "+v"(v));
    return v;
}

constexpr int kStageSlots = 3072;    // 16-byte vectors of a channel that touch the patch (forward, one block per channel)

struct TeamHeader {
    unsigned long long state;
    unsigned int done;
    unsigned int expired;
    unsigned int reserved[12];
};
constexpr unsigned long long kHeaderMagic = 0x626e7301ull << 32;   // set up
constexpr unsigned long long kHeaderBusy = 0x626e7302ull << 32;    // being set up
constexpr unsigned long long kHeaderMask = 0xffffffffull << 32;

struct FusedArgs {
    const void* x;
    const void* dy;   // backward only
    void* out;        // forward: y; backward: dx
    const float* gamma;
    const float* beta;
    float* save_mean;     // forward: written; backward: read
    float* save_invstd;
    float* running_mean;
    float* running_var;
    float* dgamma;
    float* dbeta;
    TeamHeader* hdr;            // launch counter and expired-wait count of the workspace
    unsigned long long* slots;  // [2][gridDim.x][2] words of {payload, stamp}
    IndexParams ip;
    FastDiv hwv_div, w_div;
    FastDiv wv_div;             // vectors per row (rows that are a whole number of vectors)
    int32_t rows_whole;         // W is a multiple of the vector width: no vector crosses a row
    int32_t patch_stage;        // forward, patch statistics from the registers: 1 = through the LDS staging array
    FastDiv chw_div;            // C * HW: element offset inside the tensor -> sample (pipelined kernel)
    int32_t C, W, HW;
    int32_t c0, cg;
    int32_t T, num_teams;
    uint32_t tot;   // vectors per channel: N * HW / V
    uint32_t s_cnt; // |S| per channel
    // "VDN + sampling" (Eq. 4), the MIXED flavours: samples [0, n_v) are the virtual set, `ip` describes the
    // sampled real set; mean_parts = [E_v per channel][E_s per channel] (forward: written; backward: read)
    int32_t n_v;
    float mix_beta, w_v, w_s;       // backward weights: mix_beta / s_v and (1 - mix_beta) / s_s
    double s_v;                     // n_v * HW
    float* mean_parts;
    FastDiv patch_div, pw_div;   // h_cnt * w_cnt and w_cnt of S: sampled element q -> (n, ph, pw)
    uint32_t stamp_seed;    // start of the stamp sequence if the workspace holds no launch counter yet
    uint32_t stamp_advance; // stamps this launch uses
    uint32_t spin_limit;    // polls before a missing team-mate is given up on
    int32_t mute;           // 1: members do not publish (host-forced give-up, for tests of that path)
    float eps, momentum, inv_s;
    double s;       // |S| per channel
};

// Block-wide sum of (a, b) over NT threads; result returned to every thread.
template <int NT>
__device__ __forceinline__ void block_allsum2(float& a, float& b, float* red) {
    a = wave_sum(a);
    b = wave_sum(b);
    constexpr int nw = NT / kWave;
    if (nw > 1) {
        const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
        __syncthreads();                       // red[] may still be read from the previous use
        if (lane == 0) {
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

// First stamp of this launch, the same value in every block (see TeamHeader).  In two steps, by thread 0 of every
// block of the grid: stamp_request issues the load of the header word; stamp_accept, placed behind the first
// channel's loads so that the round trip passes behind them, checks the word and leaves the stamp in the LDS word
// `word[0]` (word[1], word[2]: cleared; team_collect's flags).  No barrier: the kernels read the word (read_stamp)
// after the barrier of their first block reduction.
__device__ __forceinline__ unsigned long long stamp_request(const FusedArgs& A) {
    if (A.T == 1 || threadIdx.x != 0) return 0ull;         // single-member teams exchange nothing
    return __hip_atomic_load(&A.hdr->state, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void stamp_accept(const FusedArgs& A, unsigned long long state, uint32_t* word) {
    if (A.T == 1 || threadIdx.x != 0) return;
    TeamHeader* h = A.hdr;
    if ((state & kHeaderMask) != kHeaderMagic) {           // first use of this memory as a workspace
        bool mine = false;
        if ((state & kHeaderMask) != kHeaderBusy) {
            unsigned long long expected = state;
            mine = __hip_atomic_compare_exchange_strong(&h->state, &expected, kHeaderBusy, __ATOMIC_RELAXED,
                                                        __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (mine) {
            // a start nobody can have used here before: the host's launch count mixed with the device clock
            unsigned long long z = (static_cast<unsigned long long>(A.stamp_seed) << 32) ^ __builtin_readcyclecounter();
            z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
            z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
            state = kHeaderMagic | (z >> 32);
            __hip_atomic_store(&h->done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&h->expired, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&h->state, state, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            for (uint32_t spin = 0; spin < A.spin_limit; ++spin) {
                state = __hip_atomic_load(&h->state, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                if ((state & kHeaderMask) == kHeaderMagic) break;
                __builtin_amdgcn_s_sleep(2);
            }
        }
    }
    word[0] = uint32_t(state);
    word[1] = word[2] = 0u;
}
// Member 0 of a team (j == 0), when the team has finished its last channel: counts the team as done; the last one
// puts the next launch's first stamp and a zero count in place.
__device__ __forceinline__ void team_done(const FusedArgs& A, int j, uint32_t stamp0) {
    if (A.T == 1 || j != 0 || threadIdx.x != 0) return;
    TeamHeader* h = A.hdr;
    const unsigned int before = __hip_atomic_fetch_add(&h->done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (before + 1u == uint32_t(A.num_teams)) {
        __hip_atomic_store(&h->done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&h->state, kHeaderMagic | static_cast<unsigned long long>(stamp0 + A.stamp_advance),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}
// The stamp as a wave-uniform (scalar) value; call behind a barrier that follows draw_stamp.
__device__ __forceinline__ uint32_t read_stamp(const FusedArgs& A, const uint32_t* word) {
    if (A.T == 1) return 0u;
    return uint32_t(__builtin_amdgcn_readfirstlane(int(*static_cast<const volatile uint32_t*>(word))));
}

// Polls member `t`'s slot pair until it carries `stamp`; false (and NaN payloads) if the wait ran out.  Once a wait
// has run out in this workspace, and until the host has read the count, later waits give up after 1/64 of the polls
// (looked up every 1024 polls, so a wait that is served promptly never reads the count): the time a launch can
// spend waiting is then bounded by about one full wait rather than one per round.
__device__ __forceinline__ bool poll_pair(const FusedArgs& A, unsigned long long* theirs, uint32_t stamp, float& pa,
                                          float& pb) {
    pa = pb = __builtin_nanf("");
    uint32_t limit = A.spin_limit;
    for (uint32_t spin = 0; spin < limit; ++spin) {
        const unsigned long long wa = __hip_atomic_load(theirs, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long wb = __hip_atomic_load(theirs + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (uint32_t(wa >> 32) == stamp && uint32_t(wb >> 32) == stamp) {
            pa = __uint_as_float(uint32_t(wa));
            pb = __uint_as_float(uint32_t(wb));
            return true;
        }
        if ((spin & 1023u) == 1023u &&
            __hip_atomic_load(&A.hdr->expired, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)
            limit = A.spin_limit / 64u + 1u;
        __builtin_amdgcn_s_sleep(2);
    }
    __hip_atomic_fetch_add(&A.hdr->expired, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return false;
}

// All-gather of one (a, b) pair per team member, summed in member order in fp64, in two steps so
// that a kernel can put independent work (prefetching the next channel) between them.
// team_publish: thread 0 writes this member's stamped pair.
__device__ __forceinline__ void team_publish(const FusedArgs& A, uint32_t stamp0, int team_first_block, int j, uint32_t it,
                                             float a, float b) {
    if (A.T == 1 || threadIdx.x != 0 || A.mute) return;
    const uint32_t stamp = stamp0 + it;
    unsigned long long* mine = A.slots + (size_t(it & 1u) * gridDim.x + size_t(team_first_block + j)) * 2;
    __hip_atomic_store(mine, (static_cast<unsigned long long>(stamp) << 32) | __float_as_uint(a), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(mine + 1, (static_cast<unsigned long long>(stamp) << 32) | __float_as_uint(b), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// team_collect: waits for every member's pair and returns the team totals to every thread.  False if a wait ran
// out (the totals are then NaN).
template <int NT>
__device__ __forceinline__ bool team_collect(const FusedArgs& A, uint32_t* words, int team_first_block, uint32_t it, float a,
                                             float b, double& ta, double& tb, float* team_lds, double* bc) {
    if (A.T == 1) {
        ta = double(a);
        tb = double(b);
        return true;
    }
    const uint32_t stamp = read_stamp(A, words) + it;
    unsigned long long* base = A.slots + size_t(it & 1u) * gridDim.x * 2;
    // words[1 + (it & 1)]: set by a thread whose wait ran out in this exchange; thread 0 clears the other one, which
    // the next exchange uses, between the two barriers
    for (int t = threadIdx.x; t < A.T; t += NT) {
        float pa, pb;
        if (!poll_pair(A, base + size_t(team_first_block + t) * 2, stamp, pa, pb)) words[1 + (it & 1u)] = 1u;
        team_lds[t] = pa;
        team_lds[kMaxTeam + t] = pb;
    }
    __syncthreads();
    const bool ok = static_cast<volatile uint32_t*>(words)[1 + (it & 1u)] == 0u;
    if (threadIdx.x == 0) {
        double sa = 0.0, sb = 0.0;
        for (int t = 0; t < A.T; ++t) {
            sa += double(team_lds[t]);
            sb += double(team_lds[kMaxTeam + t]);
        }
        bc[0] = sa;
        bc[1] = sb;
        words[1 + ((it + 1u) & 1u)] = 0u;
    }
    __syncthreads();
    ta = bc[0];
    tb = bc[1];
    return ok;
}

template <int NT>
__device__ __forceinline__ bool team_allsum2(const FusedArgs& A, uint32_t* words, int team_first_block, int j, uint32_t it,
                                             float a, float b, double& ta, double& tb, float* team_lds,
                                             double* bc) {
    team_publish(A, read_stamp(A, words), team_first_block, j, it, a, b);
    return team_collect<NT>(A, words, team_first_block, it, a, b, ta, tb, team_lds, bc);
}

// Returns v unchanged but opaque to the optimiser.  Each phase of a fused kernel derives its
// addresses from its own opaque copy of the thread's first vector index, so that the compiler
// recomputes them (a few integer operations) instead of keeping KMAX 64-bit addresses alive
// across phases next to the KMAX data vectors.
__device__ __forceinline__ uint32_t opaque(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}

// Same for a data vector: stops the compiler from keeping the unpacked (wider) form of a packed
// bf16 vector alive from the reduction phase to the element-wise phase.
template <typename R>
__device__ __forceinline__ void opaque_raw(R& r) {
    asm volatile("" : "+v"(r));
}
template <>
__device__ __forceinline__ void opaque_raw<uint16_t>(uint16_t& r) {
    uint32_t t = r;
    asm volatile("" : "+v"(t));
    r = uint16_t(t);
}

// Is element (h, w) of sample n inside the box?  Whole-vector shortcuts are taken by the callers.
__device__ __forceinline__ bool in_hw(const bns_box& b, uint32_t h, uint32_t w) {
    return h >= uint32_t(b.h0) && h < uint32_t(b.h0 + b.h_cnt) && w >= uint32_t(b.w0) && w < uint32_t(b.w0 + b.w_cnt);
}

// ---------------------------------------------------------------------------------------
// sampled elements a thread reads ahead of its vectors (more: in a loop after them); registers decide how many
constexpr int patch_loads(int kmax, bool mixed) { return (kmax >= 50 || (mixed && kmax >= 16)) ? 2 : 4; }

// Offset of sampled element q of a channel from its first sampled element.
__device__ __forceinline__ size_t patch_offset(const FusedArgs& A, uint32_t q, size_t nstride) {
    const uint32_t n = fdiv(q, A.patch_div);
    const uint32_t r = q - n * A.patch_div.d;
    const uint32_t ph = fdiv(r, A.pw_div);
    return n * nstride + size_t(ph) * A.W + (r - ph * A.pw_div.d);
}

}  // namespace
}  // namespace bns
