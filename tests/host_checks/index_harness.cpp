// Host-only check of the sampling-index generator (Alg. 1, Alg. 2, Alg. 3) and of the shape / spec validation,
// meant to be built with g++ -fsanitize=address,undefined and run on a machine without a GPU.
//
//   index_harness sweep <tuples.bin> <boxes.bin>
//       tuples.bin: int64 records (N, C, H, W, mode, n_s, patch_h, patch_w, fs_per_channel, layer_id, epoch, seed, n_v),
//       n_v = 0: plain index, n_v > 0: the sampled real set of "VDN + sampling".  boxes.bin: per record int32
//       status followed by kMaxC boxes of six int32 (unused ones zero).  Every box is checked to lie inside the tensor.
//   index_harness extremes
//       every combination of extreme extents, enums and sample counts through check_shape / check_spec; whatever is
//       accepted must produce boxes inside the tensor.  Prints "accepted <n> rejected <m>".
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../paper_1810_10962_amd/csrc/bns_index.hpp"
#include "../../paper_1810_10962_amd/csrc/bns_validate.hpp"

namespace {

constexpr int kMaxC = 4;
constexpr int kFields = 13;

void die(const char* what) {
    fprintf(stderr, "index_harness: %s\n", what);
    exit(2);
}

void check_inside(const bns_box& b, const bns_shape& sh, const bns_spec& sp, int n_lo) {
    const bool ok = b.n0 >= n_lo && b.n_cnt >= 1 && int64_t(b.n0) + b.n_cnt <= sh.N && b.h0 >= 0 && b.h_cnt >= 1 &&
                    int64_t(b.h0) + b.h_cnt <= sh.H && b.w0 >= 0 && b.w_cnt >= 1 && int64_t(b.w0) + b.w_cnt <= sh.W;
    if (!ok) {
        fprintf(stderr, "box (%d %d %d %d %d %d) outside tensor %d x %d x %d, mode %d\n", b.n0, b.n_cnt, b.h0, b.h_cnt,
                b.w0, b.w_cnt, sh.N, sh.H, sh.W, int(sp.mode));
        exit(3);
    }
}

int sweep(const char* in_path, const char* out_path) {
    FILE* in = fopen(in_path, "rb");
    if (!in) die("cannot open input");
    fseek(in, 0, SEEK_END);
    const long bytes = ftell(in);
    fseek(in, 0, SEEK_SET);
    const size_t records = size_t(bytes) / (kFields * sizeof(int64_t));
    std::vector<int64_t> t(records * kFields);
    if (fread(t.data(), sizeof(int64_t), t.size(), in) != t.size()) die("short read");
    fclose(in);
    std::vector<int32_t> out(records * (1 + kMaxC * 6), 0);
    for (size_t r = 0; r < records; ++r) {
        const int64_t* f = &t[r * kFields];
        bns_shape sh = {int32_t(f[0]), int32_t(f[1]), int32_t(f[2]), int32_t(f[3]), BNS_F32, BNS_NCHW};
        bns_spec sp;
        memset(&sp, 0, sizeof sp);
        sp.mode = bns_mode(f[4]);
        sp.n_s = int32_t(f[5]);
        sp.patch_h = int32_t(f[6]);
        sp.patch_w = int32_t(f[7]);
        sp.fs_per_channel = int32_t(f[8]);
        sp.layer_id = uint32_t(f[9]);
        sp.epoch = uint32_t(f[10]);
        const uint64_t seed = uint64_t(f[11]);
        const int32_t n_v = int32_t(f[12]);
        int32_t* o = &out[r * (1 + kMaxC * 6)];
        bns::Dims d;
        bns_status s = bns::check_shape(&sh, &d);
        bns_shape real = sh;
        real.N = sh.N - n_v;
        if (s == BNS_OK) s = bns::check_spec(n_v ? &real : &sh, &sp);
        o[0] = int32_t(s);
        if (s != BNS_OK) continue;
        if (sh.C > kMaxC) die("too many channels in a record");
        const bns::IndexParams ip = n_v ? bns::make_index_params_mixed(sh, sp, seed, n_v) : bns::make_index_params(sh, sp, seed);
        for (int c = 0; c < sh.C; ++c) {
            const bns_box b = bns::box_of_channel(ip, c);
            check_inside(b, sh, sp, n_v);
            const int32_t six[6] = {b.n0, b.n_cnt, b.h0, b.h_cnt, b.w0, b.w_cnt};
            memcpy(o + 1 + c * 6, six, sizeof six);
        }
    }
    FILE* fo = fopen(out_path, "wb");
    if (!fo) die("cannot open output");
    if (fwrite(out.data(), sizeof(int32_t), out.size(), fo) != out.size()) die("short write");
    fclose(fo);
    printf("records %zu\n", records);
    return 0;
}

int extremes() {
    const int32_t ext[] = {INT32_MIN, -7, -1, 0, 1, 2, 7, 4096, 46340, 46341, 65535, 65536, 1 << 24, (1 << 24) + 1, INT32_MAX};
    const int32_t cnt[] = {INT32_MIN, -1, 0, 1, 2, 6, 7, 8, 65535, INT32_MAX};
    const int32_t enums[] = {INT32_MIN, -1, 0, 1, 2, 3, 4, 5, 6, 255, INT32_MAX};
    size_t accepted = 0, rejected = 0;
    for (int32_t N : ext)
        for (int32_t C : ext)
            for (int32_t H : ext)
                for (int32_t W : ext)
                    for (int32_t dtype : {-1, 0, 1, 2})
                        for (int32_t layout : {-1, 0, 1, 2}) {
                            bns_shape sh;
                            sh.N = N, sh.C = C, sh.H = H, sh.W = W;
                            memcpy(&sh.dtype, &dtype, sizeof dtype);      // enums may hold any bit pattern a C caller passes
                            memcpy(&sh.layout, &layout, sizeof layout);
                            bns::Dims d;
                            if (bns::check_shape(&sh, &d) != BNS_OK) {
                                ++rejected;
                                continue;
                            }
                            if (int64_t(d.HW) != int64_t(H) * W || d.vec < 1) die("Dims disagree with the shape");
                            for (int32_t mode : enums)
                                for (int32_t n_s : cnt)
                                    for (int32_t ph : cnt)
                                        for (int32_t pc : {-1, 0, 1, 2}) {
                                            bns_spec sp;
                                            memset(&sp, 0, sizeof sp);
                                            memcpy(&sp.mode, &mode, sizeof mode);
                                            sp.n_s = n_s, sp.patch_h = ph, sp.patch_w = n_s, sp.fs_per_channel = pc;
                                            sp.layer_id = 0xFFFFFFFFu, sp.epoch = uint32_t(N);
                                            if (bns::check_spec(&sh, &sp) != BNS_OK) {
                                                ++rejected;
                                                continue;
                                            }
                                            ++accepted;
                                            const bns::IndexParams ip = bns::make_index_params(sh, sp, 0xFFFFFFFFFFFFFFFFull);
                                            check_inside(bns::box_of_channel(ip, 0), sh, sp, 0);
                                            check_inside(bns::box_of_channel(ip, C - 1), sh, sp, 0);
                                        }
                        }
    // pointer helpers at the ends of the address space
    if (!bns::overlap(reinterpret_cast<void*>(16), 32, reinterpret_cast<void*>(32), 16)) die("overlap missed");
    if (bns::overlap(reinterpret_cast<void*>(16), 16, reinterpret_cast<void*>(32), 16)) die("false overlap");
    if (bns::aligned16(reinterpret_cast<void*>(UINTPTR_MAX))) die("alignment");
    printf("accepted %zu rejected %zu\n", accepted, rejected);
    return accepted > 1000 && rejected > 1000 ? 0 : 4;
}

}  // namespace

int main(int argc, char** argv) {
    if (argc == 4 && !strcmp(argv[1], "sweep")) return sweep(argv[2], argv[3]);
    if (argc == 2 && !strcmp(argv[1], "extremes")) return extremes();
    die("usage: index_harness sweep <in> <out> | index_harness extremes");
    return 1;
}
