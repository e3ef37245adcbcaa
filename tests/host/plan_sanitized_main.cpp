// Test helper (CPU): drives the host planner and the table interpreter (plan_interp.cpp) over
// cases read from a file, in a program of its own so that it can run under AddressSanitizer and
// UndefinedBehaviorSanitizer.  Every buffer has exactly the size the plan may touch (heap
// allocations, so that an access one byte outside is reported), the expected bytes come from
// the CPU oracle through the file.  Not part of the product.
//
// File: u32 ncases; per case: u32 n_tensors, u32 n_lanes, u64 chunk_bytes, u32 tile_bytes,
// u32 check_unpack; per tensor: u32 ndim, u32 dtype code, i64 shape[8], i64 strides[8],
// u64 storage bytes, storage; u64 packed bytes, expected packed (unspecified bytes 0x99);
// if check_unpack: per tensor the expected destination storage (untouched bytes 0x42).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "hxt.h"

extern "C" int plan_interp(const hxt_tensor_desc_t *descs, int n_tensors, int n_lanes, uint64_t chunk_bytes,
                           uint32_t tile_bytes, uint8_t *const *base, const uint64_t *storage_bytes,
                           uint8_t *packed, uint64_t packed_bytes, uint8_t *written, int direction,
                           int32_t *kinds_out, int32_t *uniform_out);

namespace {
bool get(FILE *f, void *p, size_t n) { return n == 0 || std::fread(p, 1, n, f) == n; }

struct Heap {                                   // exact-size heap block (size 0 still gets a valid pointer)
    uint8_t *p;
    uint64_t n;
    explicit Heap(uint64_t bytes) : p(static_cast<uint8_t *>(std::malloc(bytes ? bytes : 1))), n(bytes) {}
    ~Heap() { std::free(p); }
    Heap(const Heap &) = delete;
    Heap &operator=(const Heap &) = delete;
};
}  // namespace

int main(int argc, char **argv)
{
    if (argc != 2) return 2;
    FILE *f = std::fopen(argv[1], "rb");
    if (!f) return 2;
    uint32_t ncases = 0;
    if (!get(f, &ncases, 4)) return 2;
    for (uint32_t ci = 0; ci < ncases; ++ci) {
        uint32_t nt, k, tile, check_unpack;
        uint64_t B;
        if (!get(f, &nt, 4) || !get(f, &k, 4) || !get(f, &B, 8) || !get(f, &tile, 4) || !get(f, &check_unpack, 4)) return 2;
        std::vector<hxt_tensor_desc_t> descs(nt ? nt : 1);
        std::vector<std::vector<int64_t>> dims(2 * nt);
        std::vector<Heap *> storage, dst;
        std::vector<uint8_t *> base(nt ? nt : 1, nullptr);
        std::vector<uint64_t> sizes(nt ? nt : 1, 0);
        for (uint32_t t = 0; t < nt; ++t) {
            uint32_t ndim, code;
            int64_t shp[8], str[8];
            uint64_t sb;
            if (!get(f, &ndim, 4) || !get(f, &code, 4) || !get(f, shp, 64) || !get(f, str, 64) || !get(f, &sb, 8)) return 2;
            dims[2 * t].assign(shp, shp + ndim);               // exactly ndim entries: reading dim ndim is an overrun
            dims[2 * t + 1].assign(str, str + ndim);
            descs[t] = hxt_tensor_desc_t{int(ndim), dims[2 * t].data(), dims[2 * t + 1].data(), hxt_dtype_t(code)};
            storage.push_back(new Heap(sb));
            if (!get(f, storage.back()->p, sb)) return 2;
            sizes[t] = sb;
        }
        uint64_t pb;
        if (!get(f, &pb, 8)) return 2;
        Heap want(pb), got(pb), written(pb);
        if (!get(f, want.p, pb)) return 2;
        std::vector<int32_t> kinds(nt ? nt : 1, 0);
        int32_t uniform = 0;
        for (int direction : {0, 2}) {
            std::memset(got.p, 0x99, pb);
            std::memset(written.p, 0, pb);
            for (uint32_t t = 0; t < nt; ++t) base[t] = storage[t]->p;
            int rc = plan_interp(descs.data(), int(nt), int(k), B, tile, base.data(), sizes.data(), got.p, pb, written.p,
                                 direction, kinds.data(), &uniform);
            if (rc != 0 || std::memcmp(got.p, want.p, pb) != 0) {
                std::printf("case %u direction %d: rc %d, packed bytes %s\n", ci, direction, rc,
                            rc == 0 ? "differ from the oracle" : "not compared");
                return 1;
            }
        }
        if (check_unpack) {
            for (uint32_t t = 0; t < nt; ++t) {
                dst.push_back(new Heap(sizes[t]));
                std::memset(dst.back()->p, 0x42, sizes[t]);
                base[t] = dst.back()->p;
            }
            std::memset(written.p, 0, pb);
            int rc = plan_interp(descs.data(), int(nt), int(k), B, tile, base.data(), sizes.data(), want.p, pb, written.p, 1,
                                 kinds.data(), &uniform);
            for (uint32_t t = 0; t < nt; ++t) {
                Heap expect(sizes[t]);
                if (!get(f, expect.p, sizes[t])) return 2;
                if (rc != 0 || std::memcmp(expect.p, dst[t]->p, sizes[t]) != 0) {
                    std::printf("case %u unpack tensor %u: rc %d\n", ci, t, rc);
                    return 1;
                }
            }
        }
        for (Heap *h : storage) delete h;
        for (Heap *h : dst) delete h;
    }
    std::fclose(f);
    std::printf("plan_sanitized: ok, %u cases\n", ncases);
    return 0;
}
