// Layer-wise bit-width assigners (paper Sec. "Layer-wise Adaptive Quantization": the
// sort-and-interpolate heuristic and Algorithm 1, k-means over (size, norm) points).
// Host only; the per-layer norms they consume come from cgx_layer_sqnorms.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <vector>

#include "../../include/cgx.h"

namespace {

struct Inputs {
    std::vector<int32_t> layer;     // layers that take part (bits_in != 0, size > 0), in layer order
    std::vector<double> size, norm;
    std::vector<uint8_t> cand;      // candidate widths, ascending
};

int gather(int32_t L, const int64_t *off, const double *norms, const uint8_t *bits_in, const uint8_t *cands,
           int32_t k, uint8_t *bits_out, Inputs &in)
{
    if (L < 0 || k < 1 || k > 64) return CGX_ERR_SIZE;
    if (!cands || (L > 0 && (!off || !norms || !bits_in || !bits_out))) return CGX_ERR_NULL;
    if (L > 0 && off[0] != 0) return CGX_ERR_OFFSETS;
    for (int32_t l = 0; l < L; l++) {
        if (off[l + 1] < off[l]) return CGX_ERR_OFFSETS;
        if (bits_in[l] > 8) return CGX_ERR_BITS;
    }
    for (int32_t c = 0; c < k; c++)
        if (cands[c] < 1 || cands[c] > 8) return CGX_ERR_BITS;
    in.cand.assign(cands, cands + k);
    std::sort(in.cand.begin(), in.cand.end());
    for (int32_t l = 0; l < L; l++) {
        bits_out[l] = 0;
        if (bits_in[l] != 0 && off[l + 1] > off[l]) {
            in.layer.push_back(l);
            in.size.push_back(double(off[l + 1] - off[l]));
            in.norm.push_back(norms[l]);
        }
    }
    return CGX_OK;
}

// Scales an axis to [0, 1] by its minimum and maximum; an axis without spread becomes 0.
void unit_axis(std::vector<double> &v)
{
    const double lo = *std::min_element(v.begin(), v.end()), hi = *std::max_element(v.begin(), v.end());
    for (double &t : v) t = hi > lo ? (t - lo) / (hi - lo) : 0.0;
}

// Width of rank r among m ranked groups: the k widths spread linearly over the ranks
// (round half up); a single group takes the largest width.
uint8_t width_of_rank(int64_t r, int64_t m, const std::vector<uint8_t> &cand)
{
    const int64_t k = int64_t(cand.size());
    if (m == 1) return cand[size_t(k - 1)];
    return cand[size_t((2 * r * (k - 1) + (m - 1)) / (2 * (m - 1)))];
}

}  // namespace

extern "C" {

int cgx_assign_bits_kmeans(int32_t L, const int64_t *layer_offsets, const double *layer_norms,
                           const uint8_t *bits_in, const uint8_t *candidates, int32_t k, int32_t max_iter,
                           uint8_t *bits_out)
{
    Inputs in;
    const int rc = gather(L, layer_offsets, layer_norms, bits_in, candidates, k, bits_out, in);
    if (rc != CGX_OK) return rc;
    if (max_iter < 1) return CGX_ERR_SIZE;
    const int64_t M = int64_t(in.layer.size());
    if (M == 0) return CGX_OK;
    std::vector<double> &x = in.size, &y = in.norm;
    unit_axis(x);
    unit_axis(y);
    // points in ascending order of norm - size (ties: layer order)
    std::vector<int64_t> order(size_t(M), 0);
    std::iota(order.begin(), order.end(), int64_t(0));
    std::stable_sort(order.begin(), order.end(),
                     [&](int64_t a, int64_t b) { return y[size_t(a)] - x[size_t(a)] < y[size_t(b)] - x[size_t(b)]; });
    std::vector<int64_t> label(size_t(M), -1);
    std::vector<double> cx, cy;
    int64_t kk;
    if (M <= k) {                       // every point its own cluster
        kk = M;
        for (int64_t r = 0; r < M; r++) {
            label[size_t(order[size_t(r)])] = r;
            cx.push_back(x[size_t(order[size_t(r)])]);
            cy.push_back(y[size_t(order[size_t(r)])]);
        }
    } else {
        kk = k;
        for (int64_t c = 0; c < kk; c++) {          // start: evenly spaced ranks of that order
            const int64_t i = order[size_t(((2 * c + 1) * M) / (2 * kk))];
            cx.push_back(x[size_t(i)]);
            cy.push_back(y[size_t(i)]);
        }
        for (int32_t it = 0; it < max_iter; it++) {
            bool changed = false;
            for (int64_t i = 0; i < M; i++) {
                int64_t best = 0;
                double best_d = 0.0;
                for (int64_t c = 0; c < kk; c++) {
                    const double dx = x[size_t(i)] - cx[size_t(c)], dy = y[size_t(i)] - cy[size_t(c)];
                    const double d = dx * dx + dy * dy;
                    if (c == 0 || d < best_d) {
                        best = c;
                        best_d = d;
                    }
                }
                if (best != label[size_t(i)]) {
                    label[size_t(i)] = best;
                    changed = true;
                }
            }
            if (!changed) break;
            for (int64_t c = 0; c < kk; c++) {
                double sx = 0.0, sy = 0.0;
                int64_t cnt = 0;
                for (int64_t i = 0; i < M; i++)
                    if (label[size_t(i)] == c) {
                        sx += x[size_t(i)];
                        sy += y[size_t(i)];
                        cnt++;
                    }
                if (cnt) {                          // an empty cluster keeps its centroid
                    cx[size_t(c)] = sx / double(cnt);
                    cy[size_t(c)] = sy / double(cnt);
                }
            }
        }
    }
    // non-empty clusters ranked by centroid norm - size; widths follow the ranks
    std::vector<char> used(size_t(kk), 0);
    for (int64_t i = 0; i < M; i++) used[size_t(label[size_t(i)])] = 1;
    std::vector<int64_t> ranked;
    for (int64_t c = 0; c < kk; c++)
        if (used[size_t(c)]) ranked.push_back(c);
    std::stable_sort(ranked.begin(), ranked.end(), [&](int64_t a, int64_t b) {
        return cy[size_t(a)] - cx[size_t(a)] < cy[size_t(b)] - cx[size_t(b)];
    });
    std::vector<int64_t> rank(size_t(kk), 0);
    for (size_t r = 0; r < ranked.size(); r++) rank[size_t(ranked[r])] = int64_t(r);
    for (int64_t i = 0; i < M; i++)
        bits_out[in.layer[size_t(i)]] = width_of_rank(rank[size_t(label[size_t(i)])], int64_t(ranked.size()), in.cand);
    return CGX_OK;
}

int cgx_assign_bits_linear(int32_t L, const int64_t *layer_offsets, const double *layer_norms,
                           const uint8_t *bits_in, const uint8_t *candidates, int32_t k, uint8_t *bits_out)
{
    Inputs in;
    const int rc = gather(L, layer_offsets, layer_norms, bits_in, candidates, k, bits_out, in);
    if (rc != CGX_OK) return rc;
    const int64_t M = int64_t(in.layer.size());
    if (M == 0) return CGX_OK;
    std::vector<double> ratio(size_t(M), 0.0);
    for (int64_t i = 0; i < M; i++) ratio[size_t(i)] = in.norm[size_t(i)] / in.size[size_t(i)];
    std::vector<int64_t> order(size_t(M), 0);
    std::iota(order.begin(), order.end(), int64_t(0));
    std::stable_sort(order.begin(), order.end(),
                     [&](int64_t a, int64_t b) { return ratio[size_t(a)] < ratio[size_t(b)]; });
    for (int64_t r = 0; r < M; r++)
        bits_out[in.layer[size_t(order[size_t(r)])]] = in.cand[size_t((r * k) / M)];
    return CGX_OK;
}

int cgx_assign_buckets_from_bits(int32_t L, const uint8_t *bits_per_layer, const uint8_t *width_candidates, int32_t k,
                                 const int32_t *bucket_candidates, int32_t kb, int32_t *buckets_out)
{
    if (L < 0 || k < 1 || k > 64 || kb < 1 || kb > 64) return CGX_ERR_SIZE;
    if (!width_candidates || !bucket_candidates || (L > 0 && (!bits_per_layer || !buckets_out))) return CGX_ERR_NULL;
    std::vector<uint8_t> widths(width_candidates, width_candidates + k);
    std::vector<int32_t> sizes(bucket_candidates, bucket_candidates + kb);
    for (uint8_t w : widths)
        if (w < 1 || w > 8) return CGX_ERR_BITS;
    for (int32_t b : sizes)
        if (b < 32 || b > 8192 || b % 32) return CGX_ERR_BUCKET;
    std::sort(widths.begin(), widths.end());
    std::sort(sizes.begin(), sizes.end(), [](int32_t a, int32_t b) { return a > b; });       // longest first
    for (int32_t l = 0; l < L; l++) {
        if (bits_per_layer[l] == 0) {
            buckets_out[l] = sizes[0];
            continue;
        }
        const auto at = std::find(widths.begin(), widths.end(), bits_per_layer[l]);
        if (at == widths.end()) return CGX_ERR_BITS;        // not one of the candidates
        const int64_t i = at - widths.begin();
        buckets_out[l] = sizes[size_t(k == 1 ? 0 : (2 * i * (kb - 1) + (k - 1)) / (2 * (k - 1)))];
    }
    return CGX_OK;
}

}  // extern "C"
