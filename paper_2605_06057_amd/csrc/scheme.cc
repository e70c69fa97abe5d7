// Scheme store: text parser, built-in schemes, exact Brent verifier (paper Sec. 2.1).
#include "host_common.h"

#include <atomic>
#include <memory>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <sstream>

// Generated at build time from the text files under schemes/ (and their Kronecker
// products): const char *kBuiltinNames[], *kBuiltinTexts[]; int kBuiltinCount.
#include "builtin_schemes.inc"

namespace lcma {

static uint64_t fnv1a(uint64_t h, const void *data, size_t n) {
    const unsigned char *p = static_cast<const unsigned char *>(data);
    for (size_t i = 0; i < n; ++i) {
        h ^= p[i];
        h *= 0x100000001B3ull;
    }
    return h;
}

uint64_t scheme_hash(int m, int k, int n, int R, const int8_t *U, const int8_t *V, const int8_t *W) {
    uint64_t h = 0xCBF29CE484222325ull;
    const int dims[4] = {m, k, n, R};
    h = fnv1a(h, dims, sizeof dims);
    h = fnv1a(h, U, (size_t)R * m * k);
    h = fnv1a(h, V, (size_t)R * k * n);
    h = fnv1a(h, W, (size_t)R * m * n);
    return h;
}

// Parses the scheme text format.  Returns LCMA_OK or LCMA_ERR_PARSE (message in last error).
static lcma_status parse_text(const std::string &text, lcma_scheme *s) {
    std::vector<long> nums;
    std::istringstream in(text);
    std::string line;
    int lineno = 0;
    while (std::getline(in, line)) {
        ++lineno;
        const size_t hash = line.find('#');
        if (hash != std::string::npos) line.resize(hash);
        const char *p = line.c_str();
        while (*p) {
            while (*p == ' ' || *p == '\t' || *p == '\r' || *p == ',') ++p;
            if (!*p) break;
            char *end = nullptr;
            const long v = std::strtol(p, &end, 10);
            if (end == p) return fail(LCMA_ERR_PARSE, "scheme text: unexpected token on line %d", lineno);
            nums.push_back(v);
            p = end;
        }
    }
    if (nums.size() < 4) return fail(LCMA_ERR_PARSE, "scheme text: missing header 'm k n R'");
    const long m = nums[0], k = nums[1], n = nums[2], R = nums[3];
    if (m < 1 || k < 1 || n < 1 || R < 1 || m > 16 || k > 16 || n > 16 || R > 4096)
        return fail(LCMA_ERR_PARSE, "scheme text: grid %ld %ld %ld rank %ld out of range", m, k, n, R);
    const size_t want = 4 + (size_t)R * (m * k + k * n + m * n);
    if (nums.size() != want)
        return fail(LCMA_ERR_PARSE, "scheme text: %zu coefficients, expected %zu", nums.size() - 4, want - 4);
    for (size_t i = 4; i < nums.size(); ++i)
        if (nums[i] < -128 || nums[i] > 127)
            return fail(LCMA_ERR_PARSE, "scheme text: coefficient %ld does not fit in int8", nums[i]);
    s->m = (int)m;
    s->k = (int)k;
    s->n = (int)n;
    s->R = (int)R;
    size_t pos = 4;
    auto take = [&](std::vector<int8_t> &dst, size_t count) {
        dst.resize(count);
        for (size_t i = 0; i < count; ++i) dst[i] = (int8_t)nums[pos + i];
        pos += count;
    };
    take(s->U, (size_t)R * m * k);
    take(s->V, (size_t)R * k * n);
    take(s->W, (size_t)R * m * n);
    s->hash = scheme_hash(s->m, s->k, s->n, s->R, s->U.data(), s->V.data(), s->W.data());
    return LCMA_OK;
}

// Exact Brent identity; first_bad in row-major (i,a,b,j,c,d) order.
static bool brent_holds(const lcma_scheme *s, int64_t *first_bad) {
    const int m = s->m, k = s->k, n = s->n, R = s->R;
    // T[r][c*n+d] = W[r,c,d]; for every (i,a,b,j) form sum_r U V W over all (c,d) at once.
    std::vector<int64_t> acc((size_t)m * n);
    int64_t idx = 0;
    for (int i = 0; i < m; ++i)
        for (int a = 0; a < k; ++a)
            for (int b = 0; b < k; ++b)
                for (int j = 0; j < n; ++j) {
                    std::fill(acc.begin(), acc.end(), 0);
                    for (int r = 0; r < R; ++r) {
                        const int uv = (int)s->U[((size_t)r * m + i) * k + a] * (int)s->V[((size_t)r * k + b) * n + j];
                        if (!uv) continue;
                        const int8_t *w = &s->W[(size_t)r * m * n];
                        for (int cd = 0; cd < m * n; ++cd) acc[cd] += (int64_t)uv * w[cd];
                    }
                    for (int c = 0; c < m; ++c)
                        for (int d = 0; d < n; ++d, ++idx) {
                            const int64_t want = (a == b && i == c && j == d) ? 1 : 0;
                            if (acc[(size_t)c * n + d] != want) {
                                if (first_bad) *first_bad = idx;
                                return false;
                            }
                        }
                }
    if (first_bad) *first_bad = -1;
    return true;
}

// Built-in schemes are the ones kernels were generated for: the paper's three and every further scheme
// file that was present when the library was built (ids from 4 up).
static int builtin_index_of_id(int id) {
    for (int i = 0; i < kBuiltinCount; ++i)
        if (kBuiltinIds[i] == id) return i;
    return -1;
}

int builtin_id_of(const char *name) {
    for (int i = 0; i < kBuiltinCount; ++i)
        if (!std::strcmp(kBuiltinNames[i], name)) return kBuiltinIds[i];
    return -1;
}

const char *builtin_name_of(int id) {
    if (id == LCMA_PLAIN) return "plain";
    const int i = builtin_index_of_id(id);
    return i < 0 ? nullptr : kBuiltinNames[i];
}

int builtin_max_id() {
    int m = 0;
    for (int i = 0; i < kBuiltinCount; ++i) m = kBuiltinIds[i] > m ? kBuiltinIds[i] : m;
    return m;
}

const lcma_scheme *builtin_scheme(int id) {
    static std::vector<std::unique_ptr<lcma_scheme>> cache(kBuiltinCount); // owned: released when the library unloads
    static std::mutex mu;
    const int i = builtin_index_of_id(id);
    if (i < 0) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!cache[i]) {
        lcma_scheme *s = nullptr;
        std::string spec = std::string("builtin:") + kBuiltinNames[i];
        if (lcma_scheme_load(spec.c_str(), &s) != LCMA_OK) return nullptr;
        if (lcma_scheme_verify(s, nullptr) != LCMA_OK) {
            lcma_scheme_free(s);
            return nullptr;
        }
        cache[i].reset(s);
    }
    return cache[i].get();
}

} // namespace lcma

using namespace lcma;

extern "C" lcma_status lcma_scheme_load(const char *spec, lcma_scheme **out) {
    if (!spec || !out) return fail(LCMA_ERR_ARG, "lcma_scheme_load: null argument");
    *out = nullptr;
    std::string text;
    int builtin = 0;
    if (!std::strncmp(spec, "builtin:", 8)) {
        const char *name = spec + 8;
        int found = -1;
        for (int i = 0; i < kBuiltinCount; ++i)
            if (!std::strcmp(kBuiltinNames[i], name)) found = i;
        if (found < 0) return fail(LCMA_ERR_IO, "lcma_scheme_load: no built-in scheme named '%s'", name);
        text = kBuiltinTexts[found];
        builtin = builtin_id_of(name);
    } else {
        std::ifstream f(spec);
        if (!f) return fail(LCMA_ERR_IO, "lcma_scheme_load: cannot open '%s'", spec);
        std::stringstream ss;
        ss << f.rdbuf();
        text = ss.str();
    }
    lcma_scheme *s = new (std::nothrow) lcma_scheme();
    if (!s) return fail(LCMA_ERR_ARG, "lcma_scheme_load: out of memory");
    const lcma_status st = parse_text(text, s);
    if (st != LCMA_OK) {
        delete s;
        return st;
    }
    s->builtin = builtin > 0 ? builtin : 0;
    if (!s->builtin) { // a file holding the coefficients of a built-in scheme is that scheme
        for (int i = 0; i < kBuiltinCount; ++i) {
            const lcma_scheme *b = builtin_scheme(kBuiltinIds[i]);
            if (b && b->hash == s->hash && b->U == s->U && b->V == s->V && b->W == s->W) s->builtin = kBuiltinIds[i];
        }
    }
    *out = s;
    return LCMA_OK;
}

extern "C" lcma_status lcma_scheme_verify(const lcma_scheme *s, int64_t *first_bad) {
    if (!s) return fail(LCMA_ERR_ARG, "lcma_scheme_verify: null scheme");
    int state = s->verified.load(std::memory_order_acquire);
    if (state == 0) {
        std::lock_guard<std::mutex> lock(s->mu);
        state = s->verified.load(std::memory_order_acquire);
        if (state == 0) {
            int64_t bad = -1;
            const bool ok = brent_holds(s, &bad);
            s->first_bad = bad;
            state = ok ? 1 : 2;
            s->verified.store(state, std::memory_order_release);
        }
    }
    if (first_bad) *first_bad = s->first_bad;
    if (state == 1) return LCMA_OK;
    return fail(LCMA_ERR_BRENT, "scheme <%d,%d,%d;%d> violates Brent equation %lld", s->m, s->k, s->n, s->R,
                (long long)s->first_bad);
}

extern "C" void lcma_scheme_free(lcma_scheme *s) { delete s; }

extern "C" lcma_status lcma_scheme_info(const lcma_scheme *s, int *m, int *k, int *n, int *R, int *nnzU, int *nnzV,
                                        int *nnzW) {
    if (!s) return fail(LCMA_ERR_ARG, "lcma_scheme_info: null scheme");
    auto nnz = [](const std::vector<int8_t> &v) {
        int c = 0;
        for (int8_t x : v) c += x != 0;
        return c;
    };
    if (m) *m = s->m;
    if (k) *k = s->k;
    if (n) *n = s->n;
    if (R) *R = s->R;
    if (nnzU) *nnzU = nnz(s->U);
    if (nnzV) *nnzV = nnz(s->V);
    if (nnzW) *nnzW = nnz(s->W);
    return LCMA_OK;
}

extern "C" lcma_status lcma_scheme_coeffs(const lcma_scheme *s, int8_t *U, int8_t *V, int8_t *W) {
    if (!s || !U || !V || !W) return fail(LCMA_ERR_ARG, "lcma_scheme_coeffs: null argument");
    std::memcpy(U, s->U.data(), s->U.size());
    std::memcpy(V, s->V.data(), s->V.size());
    std::memcpy(W, s->W.data(), s->W.size());
    return LCMA_OK;
}
