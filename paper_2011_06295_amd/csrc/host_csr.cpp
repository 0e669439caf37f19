// Host side of sparse_conv_create: CSR of the pruned weights (section 7 of
// arXiv 2011.06295), the binary16 conversion of the value array (section 8) and
// the 4-bit codebook form of cluster-quantised weights (sections 6 and 9).
#include "internal.h"

#include "../../include/sparse_conv.h"

#include <algorithm>
#include <cstring>

namespace sc {

namespace {
inline uint32_t f2u(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float u2f(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }
}  // namespace

// Round-to-nearest-even float -> binary16.  Normal range: re-bias the exponent
// and add 0xfff plus the parity of the kept mantissa, so the carry performs the
// rounding; subnormal range: one float addition against 2^-1 aligns the
// mantissa so the hardware's own RNE does the work.
uint16_t float_to_half_rne(float f)
{
    const uint32_t bits = f2u(f);
    const uint16_t sign = static_cast<uint16_t>((bits >> 16) & 0x8000u);
    uint32_t a = bits & 0x7fffffffu;
    if (a > 0x7f800000u) {  // NaN: quiet, upper payload bits kept, payload never empty
        const uint32_t payload = (a >> 13) & 0x3ffu;
        return static_cast<uint16_t>(sign | 0x7e00u | (payload ? payload : 1u));
    }
    if (a >= 0x47800000u)  // |f| >= 65536 (and infinity)
        return static_cast<uint16_t>(sign | 0x7c00u);
    if (a < 0x38800000u) {  // |f| < 2^-14: result is a binary16 subnormal or zero
        const float magic = u2f(0x3f000000u);  // 0.5: ulp(0.5..1) = 2^-24 = one binary16 subnormal step
        const float shifted = u2f(a) + magic;
        return static_cast<uint16_t>(sign | (f2u(shifted) - 0x3f000000u));
    }
    const uint32_t odd = (a >> 13) & 1u;
    a += 0xc8000000u + 0xfffu + odd;  // exponent bias 127 -> 15, then round
    return static_cast<uint16_t>(sign | (a >> 13));  // a carry into 0x7c00 is the correct overflow to infinity
}

float half_to_float(uint16_t h)
{
    const uint32_t sign = (static_cast<uint32_t>(h) & 0x8000u) << 16;
    const uint32_t em = h & 0x7fffu;
    if (em >= 0x7c00u) return u2f(sign | 0x7f800000u | ((em & 0x3ffu) << 13));
    if (em < 0x0400u) {  // subnormal: em * 2^-24, exact in float
        const float v = static_cast<float>(em) * u2f(0x33800000u);
        return u2f(f2u(v) | sign);
    }
    return u2f(sign | ((em << 13) + 0x38000000u));
}

namespace {

// Which columns of every row are stored (section 7), row by row in ascending column
// order: emit(k, j, explicit_zero) is called once per stored entry.  Returns false if
// the total would not fit int32.
template <typename Emit>
bool encode_rows(const unsigned char* mask, int K, int L, bool unify, Csr& out, Emit emit)
{
    out.K = K;
    out.L = L;
    std::vector<int> count(K, 0);
    int widest = 0;
    for (int k = 0; k < K; ++k) {
        const unsigned char* m = mask + static_cast<size_t>(k) * L;
        int c = 0;
        for (int j = 0; j < L; ++j) c += (m[j] != 0);
        count[k] = c;
        widest = std::max(widest, c);
    }
    long long total = 0;
    for (int k = 0; k < K; ++k) total += unify ? widest : count[k];
    if (total >= (1ll << 31)) return false;

    out.rowptr.assign(K + 1, 0);
    out.colidx.clear();
    out.colidx.reserve(static_cast<size_t>(total));

    std::vector<unsigned char> state;  // per column of the current row: 0 dropped, 1 kept, 2 explicit zero
    for (int k = 0; k < K; ++k) {
        const unsigned char* m = mask + static_cast<size_t>(k) * L;
        state.assign(m, m + L);
        for (auto& s : state) s = s ? 1 : 0;
        if (unify) {
            int missing = widest - count[k];
            // grow stored runs to the right, left to right, newly added columns included
            for (int j = 1; j < L && missing > 0; ++j)
                if (state[j] == 0 && state[j - 1] != 0) {
                    state[j] = 2;
                    --missing;
                }
            // still short: take the lowest free columns
            for (int j = 0; j < L && missing > 0; ++j)
                if (state[j] == 0) {
                    state[j] = 2;
                    --missing;
                }
        }
        for (int j = 0; j < L; ++j) {
            if (state[j] == 0) continue;
            out.colidx.push_back(j);
            emit(k, j, state[j] == 2);
        }
        out.rowptr[k + 1] = static_cast<int>(out.colidx.size());
    }
    return true;
}

}  // namespace

bool encode_csr(const float* w, const unsigned char* mask, int K, int L, bool unify, bool half, Csr& out)
{
    out.val32.clear();
    out.coded = false;
    out.code.clear();
    if (!encode_rows(mask, K, L, unify, out, [&](int k, int j, bool zero) {
            out.val32.push_back(0.0f);
            if (!zero) std::memcpy(&out.val32.back(), w + static_cast<size_t>(k) * L + j, 4);  // bit copy: NaN payloads and -0.0 survive
        }))
        return false;
    out.val16.clear();
    if (half) {
        out.val16.resize(out.val32.size());
        for (size_t t = 0; t < out.val32.size(); ++t) {
            out.val16[t] = float_to_half_rne(out.val32[t]);
            out.val32[t] = half_to_float(out.val16[t]);
        }
    }
    return true;
}

int encode_csr_codebook(const unsigned char* index, const float* centroids, const unsigned char* mask,
                        int K, int L, bool unify, bool half, Csr& out)
{
    int zero = -1;
    float widened[16];
    for (int i = 0; i < 16; ++i) {
        out.centroid[i] = float_to_half_rne(centroids[i]);
        widened[i] = half_to_float(out.centroid[i]);
        if (zero < 0 && (out.centroid[i] & 0x7fffu) == 0) zero = i;
    }
    out.coded = true;
    out.code.clear();
    out.val32.clear();
    out.val16.clear();
    bool bad = false;
    const bool fits = encode_rows(mask, K, L, unify, out, [&](int k, int j, bool explicit_zero) {
        int c = explicit_zero ? zero : index[static_cast<size_t>(k) * L + j];
        if (c < 0 || c > 15) {
            bad = true;
            c = 0;
        }
        const size_t t = out.val32.size();
        if (t % 2 == 0) out.code.push_back(static_cast<uint8_t>(c));
        else out.code.back() = static_cast<uint8_t>(out.code.back() | (c << 4));
        out.val32.push_back(widened[c]);
        if (half) out.val16.push_back(out.centroid[c]);
    });
    if (!fits || bad) return SC_EINVAL;
    return SC_OK;
}

}  // namespace sc
