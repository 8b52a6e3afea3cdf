// access_patterns: what HBM gives for the memory access patterns a BN backward pass can have on an
// N x C x H x W tensor -- two tensors read, one written, 16-byte accesses, no arithmetic to speak of, no
// exchange between blocks.  A stand-alone program (it does not link libbns): the yardstick that the single-launch
// backward kernel is held against.  Prints one line per pattern: median and fastest time over rotating buffer
// sets, and bytes moved / median.
//
//   flat            short blocks walk memory front to back (what the streaming kernels do)
//   channel         teams of T persistent blocks take one channel at a time: member j holds chunks j, j+T, ... of
//                   the channel's N planes (K vectors per thread), loads them all, then stores them all
//                   (what "keep a channel on chip" does).  layout = real: planes C*HW apart; contiguous: the same
//                   index arithmetic on a tensor stored channel by channel; padded: planes C*HW + pad apart
//   stripes         short blocks, one vector per thread, walking stripes of G adjacent channels sample by sample
//                   (G = 1: channel by channel; G = C: flat)
//   capped          `channel` with at most CAP loads in flight per thread
//   sample-major    persistent blocks that each stream one contiguous run: the planes of G adjacent channels of
//                   one sample
//   read-only, write-only   flat passes that only load (both read tensors) or only store (the written one), with
//                   and without the non-temporal hint: what the memory gives when reads and writes do not mix
//   two passes      a read-only pass over two tensors (what a reduction does), then a pass that reads one of them
//                   again and writes a third (what the element-wise pass after it does); timed: the second pass.
//                   The first pass loads the tensor that is read again either like everything else, with the
//                   non-temporal hint, or plainly: plain loads leave it in the memory-side cache.
//
// Every pattern touches each element of the three tensors exactly once and stays inside the allocations (checked
// on the host before the launch).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef float v4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                                           \
    do {                                                                                \
        hipError_t e_ = (x);                                                            \
        if (e_ != hipSuccess) {                                                         \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);       \
            return 1;                                                                   \
        }                                                                               \
    } while (0)

namespace {

constexpr int N = 64, C = 256, HW = 56 * 56;       // the shape the benchmark's metric is quoted on, fp32
constexpr unsigned HWV = HW / 4;                   // vectors per plane
constexpr size_t kVectors = size_t(N) * C * HWV;
constexpr size_t kSpareVectorsPerSample = 65536;   // room for padded sample strides

__global__ __launch_bounds__(256) void flat_kernel(const v4* __restrict__ g, const v4* __restrict__ x, v4* __restrict__ o,
                                                    size_t n) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(g + i) * 0.5f + __builtin_nontemporal_load(x + i), o + i);
}

// read-only and write-only flat passes
template <bool NTH>
__global__ __launch_bounds__(256) void loads_kernel(const v4* __restrict__ g, const v4* __restrict__ x, float* __restrict__ out,
                                                    size_t n) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    const v4 a = NTH ? __builtin_nontemporal_load(g + i) : g[i];
    const v4 b = NTH ? __builtin_nontemporal_load(x + i) : x[i];
    if (a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w == 12345.678f) out[0] = 1.f;      // (never: keeps the loads)
}
template <bool NTH>
__global__ __launch_bounds__(256) void stores_kernel(v4* __restrict__ o, size_t n, float s) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    const v4 v = {s, s + 1.f, s + 2.f, float(threadIdx.x)};
    if (NTH) __builtin_nontemporal_store(v, o + i); else o[i] = v;
}

// two passes: first pass (g plain or non-temporal, x non-temporal), second pass (g non-temporal -> o non-temporal)
template <bool KEEP>
__global__ __launch_bounds__(256) void sums_kernel(const v4* __restrict__ g, const v4* __restrict__ x, float* __restrict__ out,
                                                   size_t n) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    const v4 a = KEEP ? g[i] : __builtin_nontemporal_load(g + i);
    const v4 b = __builtin_nontemporal_load(x + i);
    if (a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w == 12345.678f) out[0] = 1.f;      // (never: keeps the loads)
}
__global__ __launch_bounds__(256) void scale_kernel(const v4* __restrict__ g, v4* __restrict__ o, size_t n) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    __builtin_nontemporal_store(__builtin_nontemporal_load(g + i) * 2.f, o + i);
}

// layout: 0 real (sample stride `sstride` vectors), 1 channel-contiguous, 2 the real walk's arithmetic on the
// channel-contiguous addresses
struct Walk {
    int channels;        // "channels" of the walk (C / G when G adjacent channels are taken as one)
    unsigned planev;     // vectors per plane of such a channel (HWV * G)
    int T, teams, layout;
    size_t sstride;      // vectors between samples (real layout)
};

template <int NT>
__device__ __forceinline__ size_t offset_of(const Walk& w, int j, int cl, int k, unsigned tot, bool* live) {
    unsigned i = (unsigned(j) + unsigned(k) * w.T) * NT + threadIdx.x;
    *live = i < tot;
    if (i >= tot) i = tot - 1;
    if (w.layout == 1) return size_t(cl) * tot + i;
    const unsigned n = i / w.planev;
    if (w.layout == 2) return size_t(cl) * tot + size_t(n) * w.planev + (i - n * w.planev);
    return size_t(n) * w.sstride + size_t(cl) * w.planev + (i - n * w.planev);
}

template <int NT, int K, int CAP>
__global__ __launch_bounds__(NT) void channel_kernel(const v4* __restrict__ g, const v4* __restrict__ x, v4* __restrict__ o,
                                                      Walk w) {
    const int team = blockIdx.x / w.T, j = blockIdx.x % w.T;
    if (team >= w.teams) return;
    const unsigned tot = unsigned(N) * w.planev;
    for (int cl = team; cl < w.channels; cl += w.teams) {
        v4 a[K], b[K];
        bool live;
        // the first tensor's vectors, then the second's (interleaving the two is 4 % slower)
#pragma unroll
        for (int k = 0; k < K; ++k) {
            a[k] = __builtin_nontemporal_load(g + offset_of<NT>(w, j, cl, k, tot, &live));
            if (CAP == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
            if (CAP == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            if (CAP == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            b[k] = __builtin_nontemporal_load(x + offset_of<NT>(w, j, cl, k, tot, &live));
            if (CAP == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
            if (CAP == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            if (CAP == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const size_t off = offset_of<NT>(w, j, cl, k, tot, &live);
            if (live) __builtin_nontemporal_store(a[k] * 0.5f + b[k], o + off);
        }
    }
}

// block (team, n): the planes of G adjacent channels of sample n, one contiguous run of G * HWV vectors
template <int NT, int K, int G>
__global__ __launch_bounds__(NT) void sample_major_kernel(const v4* __restrict__ g, const v4* __restrict__ x,
                                                           v4* __restrict__ o, int teams) {
    const int team = blockIdx.x / N, n = blockIdx.x % N;
    if (team >= teams) return;
    constexpr unsigned run = unsigned(G) * HWV;
    static_assert(size_t(K) * NT >= run, "a block holds its run");
    for (int grp = team; grp < C / G; grp += teams) {
        const size_t base = (size_t(n) * C + size_t(grp) * G) * HWV;
        v4 a[K], b[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            unsigned i = unsigned(k) * NT + threadIdx.x;
            if (i >= run) i = run - 1;
            a[k] = __builtin_nontemporal_load(g + base + i);
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            unsigned i = unsigned(k) * NT + threadIdx.x;
            if (i >= run) i = run - 1;
            b[k] = __builtin_nontemporal_load(x + base + i);
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const unsigned i = unsigned(k) * NT + threadIdx.x;
            if (i < run) __builtin_nontemporal_store(a[k] * 0.5f + b[k], o + base + i);
        }
    }
}

bool walk_in_bounds(const Walk& w, int nt, int k) {
    const size_t tot = size_t(N) * w.planev;
    if (size_t(w.T) * nt * k < tot) return false;                                  // the team covers the channel
    if (w.layout != 0) return size_t(w.channels) * tot <= kVectors;
    const size_t last = size_t(N - 1) * w.sstride + size_t(w.channels) * w.planev; // one past the last vector touched
    return w.sstride >= size_t(w.channels) * w.planev && last <= kVectors + size_t(N) * kSpareVectorsPerSample;
}

}  // namespace

int main() {
    const size_t bytes = kVectors * sizeof(v4);
    const size_t alloc = bytes + size_t(N) * kSpareVectorsPerSample * sizeof(v4);
    constexpr int kSets = 3;
    std::vector<v4*> G(kSets), X(kSets), O(kSets);
    for (int i = 0; i < kSets; ++i) {
        CK(hipMalloc(&G[i], alloc));
        CK(hipMalloc(&X[i], alloc));
        CK(hipMalloc(&O[i], alloc));
        CK(hipMemset(G[i], 1, alloc));
        CK(hipMemset(X[i], 1, alloc));
        CK(hipMemset(O[i], 0, alloc));
    }
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    auto run = [&](const char* name, auto launch) {
        std::vector<float> ts;
        for (int it = 0; it < 30; ++it) {
            const int s = it % kSets;
            (void)hipEventRecord(e0, 0);
            launch(s);
            (void)hipEventRecord(e1, 0);
            (void)hipEventSynchronize(e1);
            float ms = 0.f;
            (void)hipEventElapsedTime(&ms, e0, e1);
            if (it >= 6) ts.push_back(ms);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            printf("%-72s launch error %s\n", name, hipGetErrorString(e));
            exit(1);
        }
        std::sort(ts.begin(), ts.end());
        const float med = ts[ts.size() / 2];
        printf("%-72s %7.1f us (fastest %6.1f)  %5.0f GB/s\n", name, med * 1e3, ts[0] * 1e3, 3.0 * bytes / med / 1e6);
        fflush(stdout);
    };
    char name[128];

    run("flat, 256-thread blocks, one vector per thread", [&](int s) {
        hipLaunchKernelGGL(flat_kernel, dim3((kVectors + 255) / 256), dim3(256), 0, 0, G[s], X[s], O[s], kVectors);
    });

#define CHANNEL(NT, K, CAP, WALK, LABEL)                                                                        \
    do {                                                                                                        \
        const Walk w_ = WALK;                                                                                   \
        if (!walk_in_bounds(w_, NT, K)) {                                                                       \
            printf("%s: walk leaves the allocation, skipped\n", LABEL);                                         \
            break;                                                                                              \
        }                                                                                                       \
        run(LABEL, [&](int s) {                                                                                 \
            hipLaunchKernelGGL((channel_kernel<NT, K, CAP>), dim3(w_.T * w_.teams), dim3(NT), 0, 0, G[s], X[s], \
                               O[s], w_);                                                                       \
        });                                                                                                     \
    } while (0)

    const size_t dense = size_t(C) * HWV;
    CHANNEL(448, 7, 0, (Walk{C, HWV, 16, 32, 0, dense}), "channel, 32 teams of 16 x 448 threads x 7 vectors, real layout");
    CHANNEL(448, 7, 0, (Walk{C, HWV, 16, 32, 1, dense}), "channel, the same, channel-contiguous layout");
    CHANNEL(448, 7, 0, (Walk{C, HWV, 16, 32, 2, dense}), "channel, the same, real walk's arithmetic on the contiguous layout");
    CHANNEL(512, 7, 0, (Walk{C, HWV, 14, 36, 0, dense}), "channel, 36 teams of 14 x 512 threads x 7 vectors, real layout");
    for (size_t pad : {size_t(64), size_t(1088), size_t(4160), size_t(32784)}) {
        snprintf(name, sizeof name, "channel, 32 x 16 x 448 x 7, sample stride padded by %zu bytes", pad * sizeof(v4));
        CHANNEL(448, 7, 0, (Walk{C, HWV, 16, 32, 0, dense + pad}), name);
    }
    CHANNEL(448, 7, 2, (Walk{C, HWV, 16, 32, 0, dense}), "capped, 32 x 16 x 448 x 7, at most 2 loads in flight per thread");
    CHANNEL(448, 7, 4, (Walk{C, HWV, 16, 32, 0, dense}), "capped, 32 x 16 x 448 x 7, at most 4 loads in flight per thread");
    CHANNEL(448, 7, 8, (Walk{C, HWV, 16, 32, 0, dense}), "capped, 32 x 16 x 448 x 7, at most 8 loads in flight per thread");
    // persistent teams that take G adjacent channels as one (team size scaled with G)
    CHANNEL(448, 7, 0, (Walk{C / 4, HWV * 4, 64, 8, 0, dense}), "channel, groups of 4 adjacent channels: 8 teams of 64 x 448 x 7");
    CHANNEL(448, 7, 0, (Walk{C / 32, HWV * 32, 512, 1, 0, dense}), "channel, groups of 32 adjacent channels: 1 team of 512 x 448 x 7");
    // short blocks, one vector per thread: stripes of G adjacent channels, sample by sample
    for (int g : {1, 2, 4, 8, 32, 64, 256}) {
        snprintf(name, sizeof name, "stripes of %d channel%s, short 256-thread blocks, one vector per thread", g, g > 1 ? "s" : "");
        const int T = 196 * g;                             // 256-thread chunks per channel of the walk
        CHANNEL(256, 1, 0, (Walk{C / g, HWV * unsigned(g), T, C / g, 0, dense}), name);
    }
    CHANNEL(256, 1, 0, (Walk{C, HWV, 196, C, 1, dense}), "stripes of 1 channel, the same, channel-contiguous layout");
#undef CHANNEL

    run("sample-major, 8 teams of 64 blocks x 448 threads, 4 channels of one sample each", [&](int s) {
        hipLaunchKernelGGL((sample_major_kernel<448, 7, 4>), dim3(N * 8), dim3(448), 0, 0, G[s], X[s], O[s], 8);
    });
    run("sample-major, 64 teams (short-lived blocks), 4 channels of one sample each", [&](int s) {
        hipLaunchKernelGGL((sample_major_kernel<448, 7, 4>), dim3(N * 64), dim3(448), 0, 0, G[s], X[s], O[s], 64);
    });
    run("sample-major, 16 teams of 64 blocks x 448 threads, 2 channels of one sample each", [&](int s) {
        hipLaunchKernelGGL((sample_major_kernel<448, 4, 2>), dim3(N * 16), dim3(448), 0, 0, G[s], X[s], O[s], 16);
    });

    float* flag = nullptr;
    CK(hipMalloc(&flag, sizeof(float)));
    {
        // (run() prints bytes of three tensors over the time: scaled here to what these passes move)
        auto timed = [&](const char* label, double tensors, auto launch) {
            std::vector<float> ts;
            for (int it = 0; it < 30; ++it) {
                (void)hipEventRecord(e0, 0);
                launch(it % kSets);
                (void)hipEventRecord(e1, 0);
                (void)hipEventSynchronize(e1);
                float ms = 0.f;
                (void)hipEventElapsedTime(&ms, e0, e1);
                if (it >= 6) ts.push_back(ms);
            }
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) {
                printf("%-72s launch error %s\n", label, hipGetErrorString(e));
                exit(1);
            }
            std::sort(ts.begin(), ts.end());
            const float med = ts[ts.size() / 2];
            printf("%-72s %7.1f us (fastest %6.1f)  %5.0f GB/s\n", label, med * 1e3, ts[0] * 1e3, tensors * bytes / med / 1e6);
            fflush(stdout);
        };
        const dim3 grid(unsigned((kVectors + 255) / 256));
        timed("read-only flat (x and dy), non-temporal loads", 2.0, [&](int s) {
            hipLaunchKernelGGL(loads_kernel<true>, grid, dim3(256), 0, 0, G[s], X[s], flag, kVectors);
        });
        timed("read-only flat (x and dy), plain loads", 2.0, [&](int s) {
            hipLaunchKernelGGL(loads_kernel<false>, grid, dim3(256), 0, 0, G[s], X[s], flag, kVectors);
        });
        timed("write-only flat (dx), non-temporal stores", 1.0, [&](int s) {
            hipLaunchKernelGGL(stores_kernel<true>, grid, dim3(256), 0, 0, O[s], kVectors, float(s));
        });
        timed("write-only flat (dx), plain stores", 1.0, [&](int s) {
            hipLaunchKernelGGL(stores_kernel<false>, grid, dim3(256), 0, 0, O[s], kVectors, float(s));
        });
    }

    // two passes over n vectors (the whole fp32 tensor, and half of it: the same tensor in bf16)
    for (size_t n : {kVectors, kVectors / 2})
        for (int keep = 0; keep < 2; ++keep) {
            std::vector<float> t1, t2;
            const dim3 grid(unsigned((n + 255) / 256));
            for (int it = 0; it < 30; ++it) {
                const int s = it % kSets;
                float ms1 = 0.f, ms2 = 0.f;
                (void)hipEventRecord(e0, 0);
                if (keep) hipLaunchKernelGGL(sums_kernel<true>, grid, dim3(256), 0, 0, G[s], X[s], flag, n);
                else hipLaunchKernelGGL(sums_kernel<false>, grid, dim3(256), 0, 0, G[s], X[s], flag, n);
                (void)hipEventRecord(e1, 0);
                (void)hipEventSynchronize(e1);
                (void)hipEventElapsedTime(&ms1, e0, e1);
                (void)hipEventRecord(e0, 0);
                hipLaunchKernelGGL(scale_kernel, grid, dim3(256), 0, 0, G[s], O[s], n);
                (void)hipEventRecord(e1, 0);
                (void)hipEventSynchronize(e1);
                (void)hipEventElapsedTime(&ms2, e0, e1);
                if (it >= 6) t1.push_back(ms1), t2.push_back(ms2);
            }
            CK(hipGetLastError());
            std::sort(t1.begin(), t1.end());
            std::sort(t2.begin(), t2.end());
            printf("two passes over %5.1f MB, first pass loads it %-17s first %6.1f us, second (read it, write as much) %6.1f us  %5.0f GB/s\n",
                   n * sizeof(v4) / 1e6, keep ? "plainly:" : "non-temporally:", t1[t1.size() / 2] * 1e3, t2[t2.size() / 2] * 1e3,
                   2.0 * n * sizeof(v4) / t2[t2.size() / 2] / 1e6);
            fflush(stdout);
        }
    return 0;
}
