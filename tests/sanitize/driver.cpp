// Host-side sanitizer driver (test infrastructure): links the library's host sources (CSR encoder,
// planner, C ABI without any kernel) and the CPU oracle into one executable built with
// -fsanitize=address,undefined, and walks random layers, geometries and launch overrides through
// create / get_csr / set_launch / rank_launches / check_plan, comparing the CSR arrays with the
// oracle's byte for byte (section 7 of arXiv 2011.06295).  Any sanitizer report or mismatch ends the
// run with a non-zero status.  No GPU call is made.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/sparse_conv.h"

extern "C" {
long long oracle_csr_rowptr(const unsigned char* mask, int K, int L, int* rowptr);
void oracle_csr_fill(const float* w, const unsigned char* mask, int K, int L, int* colidx, float* values);
int oracle_unify_mask(const unsigned char* mask, int K, int L, unsigned char* mask_out);
void oracle_to_f16_bits(const float* in, uint16_t* out, long long n);
int oracle_output_dim(int in, int pad, int filt, int stride);
}

namespace {

uint64_t state = 0x9E3779B97F4A7C15ull;
uint32_t rnd()
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (uint32_t)(state >> 32);
}
int between(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }
float unit() { return (float)(rnd() >> 8) / 16777216.0f; }

int fail(const char* what, int t)
{
    std::fprintf(stderr, "sanitize driver: %s (case %d)\n", what, t);
    return 1;
}

}  // namespace

int main()
{
    int plans = 0, cases = 0;
    for (int t = 0; t < 120; ++t) {
        const int K = between(1, 40), C = between(1, 24), R = between(1, 5), S = between(1, 5);
        const int L = C * R * S;
        const int dtype = (int)(rnd() & 1);
        const unsigned flags = (rnd() & 1) ? SC_FLAG_UNIFY_NNZ : 0u;
        const float density = (t % 7 == 0) ? 0.f : (t % 5 == 0) ? 1.f : 0.05f + 0.6f * unit();
        std::vector<float> w((size_t)K * L);
        std::vector<unsigned char> m((size_t)K * L);
        for (size_t i = 0; i < w.size(); ++i) {
            w[i] = 2.f * unit() - 1.f;
            m[i] = unit() < density ? (unsigned char)((rnd() & 1) ? 1 : 255) : 0;   // any non-zero keeps the weight
        }
        sparse_conv_t h = nullptr;
        if (sparse_conv_create(&h, w.data(), m.data(), K, C, R, S, dtype, flags) != SC_OK) return fail("create", t);
        // the oracle's CSR of the same layer
        std::vector<unsigned char> mm(m);
        for (auto& v : mm) v = v ? 1 : 0;
        if (flags) {   // the oracle's extended mask: 2 marks the explicit zeros of the unify step
            std::vector<unsigned char> m01(mm);
            oracle_unify_mask(m01.data(), K, L, mm.data());
        }
        std::vector<int> rowptr(K + 1);
        const long long nnz = oracle_csr_rowptr(mm.data(), K, L, rowptr.data());
        std::vector<int> colidx((size_t)nnz + 1);
        std::vector<float> values((size_t)nnz + 1);
        oracle_csr_fill(w.data(), mm.data(), K, L, colidx.data(), values.data());
        int gK = 0;
        long long gnnz = 0;
        const int *grp = nullptr, *gci = nullptr;
        const void* gva = nullptr;
        if (sparse_conv_get_csr(h, &gK, &gnnz, &grp, &gci, &gva) != SC_OK) return fail("get_csr", t);
        if (gK != K || gnnz != nnz) return fail("nnz differs from the oracle's", t);
        if (std::memcmp(grp, rowptr.data(), sizeof(int) * (size_t)(K + 1)) != 0) return fail("rowptr differs", t);
        if (nnz && std::memcmp(gci, colidx.data(), sizeof(int) * (size_t)nnz) != 0) return fail("colidx differs", t);
        if (dtype == SC_F16) {
            std::vector<uint16_t> bits((size_t)nnz + 1);
            oracle_to_f16_bits(values.data(), bits.data(), nnz);
            if (nnz && std::memcmp(gva, bits.data(), 2 * (size_t)nnz) != 0) return fail("binary16 values differ", t);
        } else if (nnz && std::memcmp(gva, values.data(), 4 * (size_t)nnz) != 0) {
            return fail("fp32 values differ", t);
        }
        ++cases;
        // geometries x launch overrides
        for (int g = 0; g < 4; ++g) {
            const int st = between(1, 3), pad = between(0, 3), H = between(1, 33), W = between(1, g == 0 ? 150 : 40);
            const int N = between(1, g == 1 ? 300 : 20);
            if (H + 2 * pad < R || W + 2 * pad < S) continue;
            int E = 0, F = 0;
            if (sparse_conv_output_shape(h, H, W, st, pad, &E, &F) != SC_OK) return fail("output_shape", t);
            if (E != oracle_output_dim(H, pad, R, st) || F != oracle_output_dim(W, pad, S, st)) return fail("output shape differs", t);
            static const int vs[] = {0, 1, 2, 4, 8}, kws[] = {0, 1, 2, 4, 8, 16}, lanes[] = {0, 0, 1, 2, 3, 5, 9, 17}, js[] = {0, 0, 1, 2, 4, 8};
            int params[11] = {vs[rnd() % 5], between(0, 4), between(0, 5), kws[rnd() % 6], between(0, 9), 0, between(0, 2), 0,
                              between(0, 2), lanes[rnd() % 8], js[rnd() % 6]};
            const int np = (rnd() % 3 == 0) ? 0 : 11;
            if (sparse_conv_set_launch(h, params, np) != SC_OK) continue;   // a combination the kernels do not run
            int bad = -1;
            int rc = sparse_conv_check_plan(h, N, H, W, st, pad, &bad);
            if (rc == SC_EUNSUPPORTED || rc == SC_EINVAL) continue;
            if (rc != SC_OK || bad != 0) return fail("plan check", t);
            ++plans;
            int info[16];
            if (sparse_conv_get_launch(h, N, H, W, st, pad, info) != SC_OK) return fail("get_launch", t);
            if (np == 0 && g == 2) {   // every ranked candidate can be pinned and plans consistently
                int ranked[11 * 6], count = 0;
                if (sparse_conv_rank_launches(h, N, H, W, st, pad, 6, ranked, &count) != SC_OK) return fail("rank_launches", t);
                for (int i = 0; i < count; ++i) {
                    if (sparse_conv_set_launch(h, ranked + 11 * i, 11) != SC_OK) return fail("ranked candidate refused", t);
                    if (sparse_conv_check_plan(h, N, H, W, st, pad, &bad) != SC_OK || bad != 0) return fail("ranked candidate's plan", t);
                    ++plans;
                }
            }
        }
        sparse_conv_destroy(h);
    }
    // cluster-quantised layers
    for (int t = 0; t < 20; ++t) {
        const int K = between(1, 12), C = between(1, 9), R = 3, S = 3, L = C * R * S;
        std::vector<unsigned char> idx((size_t)K * L), m((size_t)K * L);
        float cen[16];
        for (int i = 0; i < 16; ++i) cen[i] = i == 3 ? 0.f : 2.f * unit() - 1.f;
        for (size_t i = 0; i < idx.size(); ++i) {
            idx[i] = (unsigned char)(rnd() & 15);
            m[i] = unit() < 0.3f;
        }
        sparse_conv_t h = nullptr;
        if (sparse_conv_create_codebook(&h, idx.data(), cen, m.data(), K, C, R, S, (int)(rnd() & 1), (rnd() & 1) ? SC_FLAG_UNIFY_NNZ : 0u) != SC_OK)
            return fail("create_codebook", t);
        int bad = -1;
        if (sparse_conv_check_plan(h, between(1, 40), 8, 8, 1, 1, &bad) != SC_OK || bad != 0) return fail("codebook plan", t);
        ++plans;
        sparse_conv_destroy(h);
    }
    std::printf("sanitize driver: ok, %d layers byte-compared with the oracle, %d plans checked\n", cases, plans);
    return 0;
}
