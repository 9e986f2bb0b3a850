// Configuration-space encoder (Sec. 3) and q-random walk (Sec. 4.3, App. A).
#include "space.hpp"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

namespace opevo {

static thread_local std::string g_error;

void set_error(const char *fmt, ...)
{
    char buf[4096];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_error = buf;
}

const char *last_error() { return g_error.c_str(); }

static const int64_t kMaxVertices = int64_t(1) << 24;

static std::vector<int64_t> distinct_primes(int64_t n)
{
    std::vector<int64_t> ps;
    for (int64_t p = 2; p * p <= n; ++p) {
        if (n % p == 0) {
            ps.push_back(p);
            while (n % p == 0) n /= p;
        }
    }
    if (n > 1) ps.push_back(n);
    return ps;
}

// Number of ordered factorizations of C into nu factors: per prime power p^e || C the
// exponent e is spread over nu slots, binomial(e+nu-1, nu-1) ways (stars and bars).
static double count_factorizations(int64_t C, int nu)
{
    double total = 1.0;
    for (int64_t p : distinct_primes(C)) {
        int e = 0;
        for (int64_t c = C; c % p == 0; c /= p) ++e;
        double b = 1.0;
        for (int i = 1; i <= nu - 1; ++i) b = b * double(e + i) / double(i);
        total *= b;
    }
    return total;
}

// Ordered factorizations of c into `slots` factors, lexicographic (Sec. 3); `divs` are the
// divisors of the parameter's C in ascending order.
static void enum_factor(int64_t c, int slots, const std::vector<int64_t> &divs,
                        std::vector<int32_t> &prefix, std::vector<int32_t> &out, int64_t &count)
{
    if (slots == 1) {
        out.insert(out.end(), prefix.begin(), prefix.end());
        out.push_back(int32_t(c));
        ++count;
        return;
    }
    for (int64_t d : divs) {
        if (d > c) break;
        if (c % d) continue;
        prefix.push_back(int32_t(d));
        enum_factor(c / d, slots - 1, divs, prefix, out, count);
        prefix.pop_back();
    }
}

int64_t Param::index_of(const int32_t *v) const
{
    if (type == OPEVO_DISCRETE || type == OPEVO_CATEGORICAL)
        return (v[0] >= 0 && v[0] < n_verts) ? v[0] : -1;
    // FACTOR / PERMUTATION: the enumeration is lexicographically sorted
    int64_t lo = 0, hi = n_verts;
    while (lo < hi) {
        int64_t mid = (lo + hi) / 2;
        const int32_t *m = vertex(mid);
        if (std::lexicographical_compare(m, m + width, v, v + width)) lo = mid + 1;
        else hi = mid;
    }
    if (lo < n_verts && std::equal(v, v + width, vertex(lo))) return lo;
    return -1;
}

int Param::neighbors(const int32_t *v, std::vector<int32_t> &out) const
{
    int n = 0;
    switch (type) {
    case OPEVO_FACTOR:
        // move one prime z of factor s to another factor t (Sec. 3)
        for (int s = 0; s < nu; ++s) {
            for (int64_t z : distinct_primes(v[s])) {
                for (int t = 0; t < nu; ++t) {
                    if (t == s) continue;
                    size_t base = out.size();
                    out.insert(out.end(), v, v + nu);
                    out[base + s] = int32_t(v[s] / z);
                    out[base + t] = int32_t(v[t] * z);
                    ++n;
                }
            }
        }
        break;
    case OPEVO_PERMUTATION:
        // one transposition of two positions (Sec. 3)
        for (int i = 0; i < width; ++i) {
            for (int j = i + 1; j < width; ++j) {
                size_t base = out.size();
                out.insert(out.end(), v, v + width);
                std::swap(out[base + i], out[base + j]);
                ++n;
            }
        }
        break;
    case OPEVO_DISCRETE:
        // no value strictly between the two (Sec. 3): the path over the sorted values
        if (v[0] > 0) { out.push_back(v[0] - 1); ++n; }
        if (v[0] + 1 < n_values) { out.push_back(v[0] + 1); ++n; }
        break;
    case OPEVO_CATEGORICAL:
        for (int j = 0; j < n_values; ++j)
            if (j != v[0]) { out.push_back(j); ++n; }
        break;
    }
    return n;
}

void Param::walk(double q, Rng &rng, int32_t *v, std::vector<int32_t> &scratch) const
{
    for (;;) {
        scratch.clear();
        int deg = neighbors(v, scratch);
        if (deg == 0) return;                    // isolated vertex: the walk cannot move
        if (!(rng.next_double() < q)) return;    // stop with probability 1-q (Eq. 3)
        uint32_t pick = rng.next_below(uint32_t(deg));
        std::memcpy(v, scratch.data() + size_t(pick) * width, sizeof(int32_t) * width);
    }
}

static int build_param(const opevo_param_desc &d, Param &p)
{
    p.type = d.type;
    p.name = d.name ? d.name : "";
    switch (d.type) {
    case OPEVO_FACTOR: {
        if (d.nu < 1 || d.nu > 16 || d.C < 1 || d.C > INT32_MAX)
            return fail(OPEVO_E_ARG, "factor parameter needs 1 <= nu <= 16 and 1 <= C < 2^31");
        p.nu = d.nu; p.C = d.C; p.width = d.nu;
        if (count_factorizations(d.C, d.nu) > double(kMaxVertices))
            return fail(OPEVO_E_TOO_LARGE, "factor parameter C=%lld nu=%d has more than 2^24 vertices",
                        (long long)d.C, d.nu);
        std::vector<int64_t> divs;
        for (int64_t t = 1; t * t <= d.C; ++t)
            if (d.C % t == 0) { divs.push_back(t); if (t != d.C / t) divs.push_back(d.C / t); }
        std::sort(divs.begin(), divs.end());
        std::vector<int32_t> prefix;
        int64_t count = 0;
        enum_factor(d.C, d.nu, divs, prefix, p.verts, count);
        p.n_verts = count;
        break;
    }
    case OPEVO_PERMUTATION: {
        if (d.n_values < 1 || d.n_values > 10)
            return fail(OPEVO_E_ARG, "permutation parameter needs 1 <= n <= 10");
        p.n_values = d.n_values; p.width = d.n_values;
        std::vector<int32_t> perm(d.n_values);
        for (int i = 0; i < d.n_values; ++i) perm[i] = i;
        do {
            p.verts.insert(p.verts.end(), perm.begin(), perm.end());
            ++p.n_verts;
        } while (std::next_permutation(perm.begin(), perm.end()));
        break;
    }
    case OPEVO_DISCRETE: {
        if (d.n_values < 1 || !d.values) return fail(OPEVO_E_ARG, "discrete parameter needs values");
        for (int i = 0; i < d.n_values; ++i) {
            if (std::isnan(d.values[i]) || (i && !(d.values[i - 1] < d.values[i])))
                return fail(OPEVO_E_ARG, "discrete values must be strictly ascending");
        }
        p.n_values = d.n_values; p.width = 1; p.n_verts = d.n_values;
        p.values.assign(d.values, d.values + d.n_values);
        for (int i = 0; i < d.n_values; ++i) p.verts.push_back(i);
        break;
    }
    case OPEVO_CATEGORICAL: {
        if (d.n_values < 1) return fail(OPEVO_E_ARG, "categorical parameter needs n_values >= 1");
        p.n_values = d.n_values; p.width = 1; p.n_verts = d.n_values;
        for (int i = 0; i < d.n_values; ++i) p.verts.push_back(i);
        break;
    }
    default:
        return fail(OPEVO_E_ARG, "unknown parameter type %d", d.type);
    }
    return OPEVO_OK;
}

int make_space(const opevo_param_desc *params, int n_params, opevo_space **out)
{
    if (!params || n_params < 1 || !out) return fail(OPEVO_E_ARG, "space_create: bad arguments");
    opevo_space *sp = new (std::nothrow) opevo_space;
    if (!sp) return fail(OPEVO_E_ARG, "out of memory");
    sp->params.resize(n_params);
    int off = 0;
    for (int i = 0; i < n_params; ++i) {
        int rc = build_param(params[i], sp->params[i]);
        if (rc != OPEVO_OK) { delete sp; return rc; }
        sp->params[i].offset = off;
        off += sp->params[i].width;
    }
    sp->width = off;
    *out = sp;
    return OPEVO_OK;
}

}  // namespace opevo

using namespace opevo;

bool opevo_space::is_legal(const int32_t *cfg) const
{
    for (const Param &p : params)
        if (p.index_of(cfg + p.offset) < 0) return false;
    return true;
}

double opevo_space::size() const
{
    double n = 1.0;
    for (const Param &p : params) n *= double(p.n_verts);
    return n;
}

bool opevo_space::rankable() const { return size() < 4.0e18; }

int64_t opevo_space::rank(const int32_t *cfg) const
{
    int64_t r = 0;
    for (const Param &p : params) {
        int64_t i = p.index_of(cfg + p.offset);
        if (i < 0) return -1;
        r = r * p.n_verts + i;
    }
    return r;
}

void opevo_space::unrank(int64_t r, int32_t *cfg) const
{
    for (size_t k = params.size(); k-- > 0;) {
        const Param &p = params[k];
        std::memcpy(cfg + p.offset, p.vertex(r % p.n_verts), sizeof(int32_t) * p.width);
        r /= p.n_verts;
    }
}

void opevo_space::random(Rng &rng, int32_t *cfg) const
{
    for (const Param &p : params) {
        uint32_t i = rng.next_below(uint32_t(p.n_verts));
        std::memcpy(cfg + p.offset, p.vertex(i), sizeof(int32_t) * p.width);
    }
}

void opevo_space::mutate(double q, Rng &rng, int32_t *cfg) const
{
    std::vector<int32_t> scratch;
    for (const Param &p : params) p.walk(q, rng, cfg + p.offset, scratch);
}

void opevo_space::mutate_uniform(double q, Rng &rng, int32_t *cfg) const
{
    for (const Param &p : params) {
        if (!(rng.next_double() < q)) continue;
        uint32_t i = rng.next_below(uint32_t(p.n_verts));
        std::memcpy(cfg + p.offset, p.vertex(i), sizeof(int32_t) * p.width);
    }
}

// ------------------------------------------------------------------------------ C ABI
extern "C" {

const char *opevo_last_error(void) { return opevo::last_error(); }

const char *opevo_version(void) { return "opevo-gfx950 0.1"; }

const char *opevo_status_name(int status)
{
    switch (status) {
    case OPEVO_OK: return "OK";
    case OPEVO_E_ARG: return "E_ARG";
    case OPEVO_E_ILLEGAL: return "E_ILLEGAL";
    case OPEVO_E_INVALID: return "E_INVALID";
    case OPEVO_E_HIPRTC: return "E_HIPRTC";
    case OPEVO_E_HIP: return "E_HIP";
    case OPEVO_E_PARITY: return "E_PARITY";
    case OPEVO_E_TOO_LARGE: return "E_TOO_LARGE";
    case OPEVO_E_STATE: return "E_STATE";
    default: return "E_UNKNOWN";
    }
}

int opevo_rng_create(uint64_t seed, opevo_rng **out)
{
    if (!out) return fail(OPEVO_E_ARG, "rng_create: out is NULL");
    *out = new (std::nothrow) opevo_rng(seed);
    return *out ? OPEVO_OK : fail(OPEVO_E_ARG, "out of memory");
}

int opevo_rng_destroy(opevo_rng *rng) { delete rng; return OPEVO_OK; }

int opevo_rng_next_u64(opevo_rng *rng, uint64_t *out)
{
    if (!rng || !out) return fail(OPEVO_E_ARG, "rng_next_u64: NULL argument");
    *out = rng->rng.next_u64();
    return OPEVO_OK;
}

int opevo_rng_next_double(opevo_rng *rng, double *out)
{
    if (!rng || !out) return fail(OPEVO_E_ARG, "rng_next_double: NULL argument");
    *out = rng->rng.next_double();
    return OPEVO_OK;
}

int opevo_rng_next_below(opevo_rng *rng, uint32_t n, uint32_t *out)
{
    if (!rng || !out || n == 0) return fail(OPEVO_E_ARG, "rng_next_below: NULL argument or n == 0");
    *out = rng->rng.next_below(n);
    return OPEVO_OK;
}

int opevo_space_create(const opevo_param_desc *params, int n_params, opevo_space **out)
{
    return opevo::make_space(params, n_params, out);
}

int opevo_space_destroy(opevo_space *space) { delete space; return OPEVO_OK; }

int opevo_space_num_params(const opevo_space *space, int *n_params)
{
    if (!space || !n_params) return fail(OPEVO_E_ARG, "space_num_params: NULL argument");
    *n_params = int(space->params.size());
    return OPEVO_OK;
}

int opevo_space_width(const opevo_space *space, int *n_int32)
{
    if (!space || !n_int32) return fail(OPEVO_E_ARG, "space_width: NULL argument");
    *n_int32 = space->width;
    return OPEVO_OK;
}

#define CHECK_PARAM(fn)                                                             \
    if (!space) return fail(OPEVO_E_ARG, fn ": space is NULL");                     \
    if (param < 0 || param >= int(space->params.size()))                            \
        return fail(OPEVO_E_ARG, fn ": parameter index %d out of range", param);    \
    const Param &p = space->params[param];

int opevo_space_param_slice(const opevo_space *space, int param, int *offset, int *width)
{
    CHECK_PARAM("space_param_slice")
    if (offset) *offset = p.offset;
    if (width) *width = p.width;
    return OPEVO_OK;
}

int opevo_space_param_name(const opevo_space *space, int param, const char **name)
{
    CHECK_PARAM("space_param_name")
    if (!name) return fail(OPEVO_E_ARG, "space_param_name: name is NULL");
    *name = p.name.c_str();
    return OPEVO_OK;
}

int opevo_space_param_size(const opevo_space *space, int param, int64_t *n_vertices)
{
    CHECK_PARAM("space_param_size")
    if (!n_vertices) return fail(OPEVO_E_ARG, "space_param_size: NULL argument");
    *n_vertices = p.n_verts;
    return OPEVO_OK;
}

int opevo_space_size(const opevo_space *space, double *n_configs)
{
    if (!space || !n_configs) return fail(OPEVO_E_ARG, "space_size: NULL argument");
    *n_configs = space->size();
    return OPEVO_OK;
}

int opevo_space_is_legal(const opevo_space *space, const int32_t *cfg)
{
    if (!space || !cfg) return fail(OPEVO_E_ARG, "space_is_legal: NULL argument");
    return space->is_legal(cfg) ? OPEVO_OK : fail(OPEVO_E_ILLEGAL, "configuration is not in the space");
}

int opevo_space_enumerate(const opevo_space *space, int param, int32_t *out,
                          int64_t cap_vertices, int64_t *n)
{
    CHECK_PARAM("space_enumerate")
    if (n) *n = p.n_verts;
    if (!out || cap_vertices < p.n_verts)
        return fail(OPEVO_E_ARG, "space_enumerate: capacity %lld < %lld vertices",
                    (long long)cap_vertices, (long long)p.n_verts);
    std::memcpy(out, p.verts.data(), sizeof(int32_t) * p.verts.size());
    return OPEVO_OK;
}

int opevo_space_neighbors(const opevo_space *space, int param, const int32_t *v,
                          int32_t *out, int cap_vertices, int *n)
{
    CHECK_PARAM("space_neighbors")
    if (!v || !n) return fail(OPEVO_E_ARG, "space_neighbors: NULL argument");
    if (p.index_of(v) < 0) return fail(OPEVO_E_ILLEGAL, "space_neighbors: not a vertex of parameter %d", param);
    std::vector<int32_t> nb;
    *n = p.neighbors(v, nb);
    if (*n > cap_vertices || (!out && *n > 0))
        return fail(OPEVO_E_ARG, "space_neighbors: capacity %d < %d neighbours", cap_vertices, *n);
    if (*n) std::memcpy(out, nb.data(), sizeof(int32_t) * nb.size());
    return OPEVO_OK;
}

int opevo_space_rank(const opevo_space *space, const int32_t *cfg, int64_t *rank)
{
    if (!space || !cfg || !rank) return fail(OPEVO_E_ARG, "space_rank: NULL argument");
    if (!space->rankable()) return fail(OPEVO_E_TOO_LARGE, "space_rank: space has 2^62 members or more");
    *rank = space->rank(cfg);
    return *rank >= 0 ? OPEVO_OK : fail(OPEVO_E_ILLEGAL, "configuration is not in the space");
}

int opevo_space_unrank(const opevo_space *space, int64_t rank, int32_t *cfg_out)
{
    if (!space || !cfg_out) return fail(OPEVO_E_ARG, "space_unrank: NULL argument");
    if (!space->rankable()) return fail(OPEVO_E_TOO_LARGE, "space_unrank: space has 2^62 members or more");
    if (rank < 0 || double(rank) >= space->size()) return fail(OPEVO_E_ARG, "space_unrank: rank out of range");
    space->unrank(rank, cfg_out);
    return OPEVO_OK;
}

int opevo_space_random(const opevo_space *space, opevo_rng *rng, int32_t *cfg_out)
{
    if (!space || !rng || !cfg_out) return fail(OPEVO_E_ARG, "space_random: NULL argument");
    space->random(rng->rng, cfg_out);
    return OPEVO_OK;
}

static int check_q(double q)
{
    if (!(q >= 0.0 && q < 1.0)) return fail(OPEVO_E_ARG, "mutation rate q must satisfy 0 <= q < 1");
    return OPEVO_OK;
}

int opevo_space_walk(const opevo_space *space, int param, double q, opevo_rng *rng, int32_t *v)
{
    CHECK_PARAM("space_walk")
    if (!rng || !v) return fail(OPEVO_E_ARG, "space_walk: NULL argument");
    if (int rc = check_q(q)) return rc;
    if (p.index_of(v) < 0) return fail(OPEVO_E_ILLEGAL, "space_walk: not a vertex of parameter %d", param);
    std::vector<int32_t> scratch;
    p.walk(q, rng->rng, v, scratch);
    return OPEVO_OK;
}

int opevo_space_mutate(const opevo_space *space, double q, opevo_rng *rng, int32_t *cfg_inout)
{
    if (!space || !rng || !cfg_inout) return fail(OPEVO_E_ARG, "space_mutate: NULL argument");
    if (int rc = check_q(q)) return rc;
    if (!space->is_legal(cfg_inout)) return fail(OPEVO_E_ILLEGAL, "space_mutate: configuration is not in the space");
    space->mutate(q, rng->rng, cfg_inout);
    return OPEVO_OK;
}

int opevo_qrw_exact(const opevo_space *space, int param, const int32_t *start, double q,
                    double *probs_out, int64_t cap)
{
    CHECK_PARAM("qrw_exact")
    if (!start || !probs_out) return fail(OPEVO_E_ARG, "qrw_exact: NULL argument");
    if (int rc = check_q(q)) return rc;
    const int64_t n = p.n_verts;
    if (n > 2048) return fail(OPEVO_E_TOO_LARGE, "qrw_exact: %lld vertices > 2048", (long long)n);
    if (cap < n) return fail(OPEVO_E_ARG, "qrw_exact: capacity %lld < %lld", (long long)cap, (long long)n);
    const int64_t s = p.index_of(start);
    if (s < 0) return fail(OPEVO_E_ILLEGAL, "qrw_exact: start is not a vertex of parameter %d", param);

    // A = I - Q with Q[v][u] = q/|S(u)| for v in S(u) (Eq. 3; App. A)
    std::vector<double> A(size_t(n) * n, 0.0), rhs(n, 0.0);
    std::vector<int32_t> nb;
    for (int64_t u = 0; u < n; ++u) {
        A[u * n + u] = 1.0;
        nb.clear();
        int deg = p.neighbors(p.vertex(u), nb);
        for (int k = 0; k < deg; ++k) {
            int64_t v = p.index_of(nb.data() + size_t(k) * p.width);
            A[v * n + u] -= q / deg;
        }
        if (u == s && deg == 0) {   // isolated start: point mass
            for (int64_t i = 0; i < n; ++i) probs_out[i] = (i == s) ? 1.0 : 0.0;
            return OPEVO_OK;
        }
    }
    rhs[s] = 1.0 - q;
    // Gaussian elimination with partial pivoting, then back substitution.
    for (int64_t c = 0; c < n; ++c) {
        int64_t piv = c;
        for (int64_t r = c + 1; r < n; ++r)
            if (std::fabs(A[r * n + c]) > std::fabs(A[piv * n + c])) piv = r;
        if (A[piv * n + c] == 0.0) return fail(OPEVO_E_ARG, "qrw_exact: singular system");
        if (piv != c) {
            for (int64_t j = 0; j < n; ++j) std::swap(A[c * n + j], A[piv * n + j]);
            std::swap(rhs[c], rhs[piv]);
        }
        for (int64_t r = c + 1; r < n; ++r) {
            double f = A[r * n + c] / A[c * n + c];
            if (f == 0.0) continue;
            for (int64_t j = c; j < n; ++j) A[r * n + j] -= f * A[c * n + j];
            rhs[r] -= f * rhs[c];
        }
    }
    for (int64_t r = n; r-- > 0;) {
        double acc = rhs[r];
        for (int64_t j = r + 1; j < n; ++j) acc -= A[r * n + j] * probs_out[j];
        probs_out[r] = acc / A[r * n + r];
    }
    return OPEVO_OK;
}

}  // extern "C"
