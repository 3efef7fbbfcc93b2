// Host-only exerciser for a build with -fsanitize=address,undefined: the plan code of the library
// (validation, sizes, tile tables), its bit-width assigners, and the CPU oracle, on plans with every
// kind of layer.  Any out-of-bounds access, overflow or misaligned access aborts the run; the
// invariants checked here make it fail with a message.  Test infrastructure: links the oracle.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../../include/cgx.h"
#include "../../paper_2111_08617_amd/csrc/cgx_plan.h"

extern "C" {
int oracle_sizes(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int32_t dt,
                 uint64_t *packed_bytes, uint64_t *meta_bytes);
int oracle_quantize(const void *grad, int64_t n, int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket,
                    uint64_t seed, int32_t dt, uint8_t *packed, float *meta);
int oracle_dequant_reduce(const uint8_t *const *packed, const float *const *meta, int32_t W, int64_t n, int32_t L,
                          const int64_t *off, const uint8_t *bits, int32_t bucket, int32_t dt, float *sum32,
                          double *sum64, double *abs64);
int oracle_unpack_codes(const uint8_t *packed, int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                        int32_t bucket, int32_t dt, uint8_t *codes);
int oracle_qsgd_sizes(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int32_t dt,
                      uint64_t *packed_bytes, uint64_t *meta_bytes);
int oracle_qsgd_quantize(const void *grad, int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                         int32_t bucket, uint64_t seed, int32_t dt, uint8_t *packed, float *meta);
int oracle_qsgd_dequant_reduce(const uint8_t *const *packed, const float *const *meta, int32_t W, int64_t n,
                               int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int32_t dt,
                               float *sum32, double *sum64, double *abs64);
void oracle_float_to_half(const float *in, int64_t count, uint16_t *out);
int oracle_layer_sqnorms(const void *buf, int64_t n, int32_t L, const int64_t *off, int32_t dt, double *out);
}

#define CHECK(cond)                                                                 \
    do {                                                                            \
        if (!(cond)) {                                                              \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                           \
        }                                                                           \
    } while (0)

struct Plan {
    std::vector<int64_t> off;
    std::vector<uint8_t> bits;
    int64_t n() const { return off.back(); }
    int32_t L() const { return int32_t(bits.size()); }
};

static Plan edge_plan(int bucket, std::mt19937 &rng)
{
    // every width, pass-through layers, empty layers, layers shorter than a bucket, ragged ends, whole
    // chunks, layers that start on odd elements
    const int sizes[] = {5000, 37, 0, 64, 4096 + 13, 1, 8 * bucket, 2 * bucket + 31, 1000, 3, 12345, 777, 2048, 8192 * 2, 1024};
    const int widths[] = {4, 0, 3, 2, 8, 5, 1, 3, 0, 4, 6, 7, 2, 4, 8};
    Plan p;
    p.off.push_back(0);
    for (size_t i = 0; i < sizeof(sizes) / sizeof(sizes[0]); i++) {
        p.off.push_back(p.off.back() + sizes[i] + int(rng() % 3 == 0));
        p.bits.push_back(uint8_t(widths[i]));
    }
    return p;
}

static void check_tiles(const Plan &p, int bucket, int dt, int chunk, int chunks_per_tile, const int32_t *layer_buckets)
{
    using namespace cgx;
    CHECK(validate_plan(p.n(), p.L(), p.off.data(), p.bits.data(), bucket, dt) == CGX_OK);
    const PlanShape shape = plan_shape(p.L(), p.off.data(), p.bits.data(), bucket, dt, layer_buckets);
    std::vector<int> covered(size_t(p.n()), 0);
    // a plan with a bucket size per layer takes one table per lane mapping in use
    const int classes[3] = {32, 128, 8192};
    size_t total_tiles = 0;
    for (int c = 0; c < (layer_buckets ? 3 : 1); c++) {
        const int launch_bucket = layer_buckets ? classes[c] : bucket;
        if (layer_buckets && mapping_of(launch_bucket, chunk) != c + (c == 0 ? 1 : c == 1 ? -1 : 0)) continue;
        std::vector<Tile> tiles;
        std::vector<uint32_t> slots;
        std::vector<int64_t> first;
        build_tiles(p.L(), p.off.data(), p.bits.data(), launch_bucket, dt, chunk, chunks_per_tile, tiles, &slots, &first,
                    layer_buckets, c == 0);
        CHECK(slots.size() == tiles.size() && first.size() == size_t(p.L()) + 1);
        total_tiles += tiles.size();
        std::vector<char> slot_used(tiles.size(), 0);
        for (size_t t = 0; t < tiles.size(); t++) {
            const Tile &tile = tiles[t];
            CHECK(tile.count > 0 && tile.elem0 >= 0 && tile.elem0 + tile.count <= p.n());
            for (uint32_t j = 0; j < tile.count; j++) covered[size_t(tile.elem0 + j)]++;
            const uint32_t b = tile_bits(tile);
            const uint64_t payload = b ? (uint64_t(tile.count) * b + 7) / 8 : uint64_t(tile.count) * (dt == CGX_F16 ? 2 : 4);
            CHECK(tile.packed_off >= 0 && uint64_t(tile.packed_off) + payload + tile.pad <= shape.packed_bytes);
            if (b) {
                const int own = tile_bucket(tile);
                CHECK(own >= 32 && own % 32 == 0);
                CHECK(uint64_t(tile.bucket0) + (tile.count + own - 1) / own <= shape.n_buckets);
                if (is_vector_kind(tile_kind(tile))) CHECK(tile.count % uint32_t(chunk) == 0 || tile_kind(tile) == kQuantWide);
            }
            CHECK(slots[t] < tiles.size() && !slot_used[slots[t]]);
            slot_used[slots[t]] = 1;
        }
    }
    CHECK(total_tiles > 0);
    for (int64_t i = 0; i < p.n(); i++) CHECK(covered[size_t(i)] == 1);    // the tables together: every element once
}

static void check_oracle(const Plan &p, int bucket, int dt, std::mt19937 &rng)
{
    std::normal_distribution<float> normal(0.0f, 1.0f);
    const int64_t n = p.n();
    std::vector<float> x(size_t(n) + 1);
    for (auto &v : x) v = normal(rng) * 0.01f;
    std::vector<uint16_t> h(size_t(n) + 1);
    oracle_float_to_half(x.data(), n, h.data());
    const void *grad = dt == CGX_F16 ? static_cast<const void *>(h.data()) : static_cast<const void *>(x.data());
    uint64_t pb = 0, mb = 0;
    CHECK(oracle_sizes(n, p.L(), p.off.data(), p.bits.data(), bucket, dt, &pb, &mb) == 0);
    const cgx::PlanShape shape = cgx::plan_shape(p.L(), p.off.data(), p.bits.data(), bucket, dt);
    CHECK(shape.packed_bytes == pb && shape.meta_bytes == mb);           // the library's sizes are the oracle's
    // exactly sized buffers: a write past the end is an error the sanitizer reports
    std::vector<std::vector<uint8_t>> packed(3, std::vector<uint8_t>(pb));
    std::vector<std::vector<float>> meta(3, std::vector<float>(mb / 4));
    const uint8_t *pp[3];
    const float *mp[3];
    for (int w = 0; w < 3; w++) {
        CHECK(oracle_quantize(grad, n, p.L(), p.off.data(), p.bits.data(), bucket, 100 + w, dt, packed[w].data(),
                              meta[w].data()) == 0);
        pp[w] = packed[w].data();
        mp[w] = meta[w].data();
    }
    std::vector<uint8_t> codes(static_cast<size_t>(n));
    CHECK(oracle_unpack_codes(pp[0], n, p.L(), p.off.data(), p.bits.data(), bucket, dt, codes.data()) == 0);
    for (int32_t l = 0; l < p.L(); l++)
        for (int64_t i = p.off[l]; i < p.off[l + 1]; i++)
            CHECK(p.bits[l] ? codes[size_t(i)] < (1u << p.bits[l]) : codes[size_t(i)] == 0xff);
    std::vector<float> s32(static_cast<size_t>(n));
    std::vector<double> s64(static_cast<size_t>(n)), a64(static_cast<size_t>(n));
    CHECK(oracle_dequant_reduce(pp, mp, 3, n, p.L(), p.off.data(), p.bits.data(), bucket, dt, s32.data(), s64.data(),
                                a64.data()) == 0);
    for (int64_t i = 0; i < n; i++) CHECK(std::fabs(double(s32[size_t(i)]) - s64[size_t(i)]) <= 1e-6 * a64[size_t(i)] + 1e-45);
    std::vector<double> sq(size_t(p.L()));
    CHECK(oracle_layer_sqnorms(grad, n, p.L(), p.off.data(), dt, sq.data()) == 0);
    // norm-and-sign form (no 1-bit layers)
    Plan q = p;
    for (auto &b : q.bits) b = b == 1 ? 2 : b;
    uint64_t qpb = 0, qmb = 0;
    CHECK(oracle_qsgd_sizes(n, q.L(), q.off.data(), q.bits.data(), bucket, dt, &qpb, &qmb) == 0);
    std::vector<uint8_t> qp(qpb);
    std::vector<float> qm(qmb / 4);
    CHECK(oracle_qsgd_quantize(grad, n, q.L(), q.off.data(), q.bits.data(), bucket, 7, dt, qp.data(), qm.data()) == 0);
    const uint8_t *qpp[1] = {qp.data()};
    const float *qmp[1] = {qm.data()};
    CHECK(oracle_qsgd_dequant_reduce(qpp, qmp, 1, n, q.L(), q.off.data(), q.bits.data(), bucket, dt, s32.data(),
                                     s64.data(), a64.data()) == 0);
}

static void check_assigners(const Plan &p, std::mt19937 &rng)
{
    std::uniform_real_distribution<double> uni(0.0, 10.0);
    std::vector<double> norms(size_t(p.L()));
    for (auto &v : norms) v = uni(rng);
    const uint8_t cands[4] = {8, 2, 4, 3};
    std::vector<uint8_t> out(size_t(p.L()), 0xee);
    for (int k = 1; k <= 4; k++) {
        CHECK(cgx_assign_bits_kmeans(p.L(), p.off.data(), norms.data(), p.bits.data(), cands, k, 50, out.data()) == CGX_OK);
        for (int32_t l = 0; l < p.L(); l++) {
            const bool takes_part = p.bits[l] != 0 && p.off[l + 1] > p.off[l];
            bool is_cand = false;
            for (int c = 0; c < k; c++) is_cand |= out[size_t(l)] == cands[c];
            CHECK(takes_part ? is_cand : out[size_t(l)] == 0);
        }
        CHECK(cgx_assign_bits_linear(p.L(), p.off.data(), norms.data(), p.bits.data(), cands, k, out.data()) == CGX_OK);
        const int32_t sizes[3] = {128, 1024, 4096};
        std::vector<int32_t> buckets(size_t(p.L()), -1);
        CHECK(cgx_assign_buckets_from_bits(p.L(), out.data(), cands, k, sizes, 3, buckets.data()) == CGX_OK);
        for (int32_t b : buckets) CHECK(b == 128 || b == 1024 || b == 4096);
    }
    CHECK(cgx_assign_bits_kmeans(p.L(), p.off.data(), norms.data(), p.bits.data(), cands, 0, 50, out.data()) == CGX_ERR_SIZE);
}

int main()
{
    std::mt19937 rng(12345);
    const int buckets[] = {32, 64, 96, 128, 512, 1024, 2048, 4096, 8192, 8160};
    int plans = 0;
    for (int bucket : buckets) {
        const Plan p = edge_plan(bucket, rng);
        for (int dt : {int(CGX_F32), int(CGX_F16)}) {
            for (int chunk : {1024, 2048})
                for (int cpt : {1, 3}) check_tiles(p, bucket, dt, chunk, cpt, nullptr);
            check_oracle(p, bucket, dt, rng);
            plans++;
        }
        std::vector<int32_t> per_layer(size_t(p.L()));
        for (auto &b : per_layer) b = buckets[rng() % 10];
        CHECK(cgx::validate_layer_buckets(p.L(), per_layer.data()) == CGX_OK);
        for (int chunk : {1024, 2048}) check_tiles(p, 32, CGX_F32, chunk, 1, per_layer.data());
        check_assigners(p, rng);
    }
    // rejected plans stay rejected without touching anything
    const int64_t bad_off[3] = {0, 10, 5};
    const uint8_t two_bits[2] = {4, 4};
    CHECK(cgx::validate_plan(5, 2, bad_off, two_bits, 128, CGX_F32) == CGX_ERR_OFFSETS);
    CHECK(cgx::validate_plan(5, 2, nullptr, two_bits, 128, CGX_F32) == CGX_ERR_NULL);
    std::printf("host sanitize driver: %d plans, all checks passed\n", plans);
    return 0;
}
