// Symbol side of the operators (Sec. 3.1.2): everything that depends only on the symbols and the
// user function, computed once on the host for the whole batch and uploaded as index arrays.
#include "internal.h"

#include <algorithm>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <set>
#include <unordered_map>

namespace dol {

// ---------------------------------------------------------------- errors

static thread_local std::string g_last_error;

void set_error(const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
}

dol_status fail(dol_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return st;
}

dol_status hip_fail(hipError_t e, const char *what)
{
    set_error("%s: %s", what, hipGetErrorString(e));
    return e == hipErrorOutOfMemory ? DOL_ENOMEM : DOL_EHIP;
}

hipError_t allow_dynamic_lds(const void *kernel, size_t bytes)
{
    static std::mutex mu;
    static std::set<std::pair<int, const void *>> *seen = new std::set<std::pair<int, const void *>>;   // never destroyed
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (seen->count({dev, kernel})) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
    if (e == hipSuccess) seen->insert({dev, kernel});
    return e;
}

// ---------------------------------------------------------------- function tables

struct Tuple {
    int32_t i, j, id;
};

static dol_status build_table(int32_t na, int32_t nb, std::vector<Tuple> &tup, dol_fn_table **out)
{
    // ascending (i, j); a function has one value per argument tuple
    std::sort(tup.begin(), tup.end(), [](const Tuple &x, const Tuple &y) { return x.i != y.i ? x.i < y.i : x.j < y.j; });
    for (size_t t = 1; t < tup.size(); ++t)
        if (tup[t].i == tup[t - 1].i && tup[t].j == tup[t - 1].j)
            return fail(DOL_EINVAL, "function table lists the tuple (%d, %d) twice", tup[t].i, tup[t].j);

    std::unique_ptr<dol_fn_table> tb(new (std::nothrow) dol_fn_table);
    if (!tb) return fail(DOL_ENOMEM, "out of host memory");
    tb->na = na;
    tb->nb = nb;
    tb->n_tuples = static_cast<int64_t>(tup.size());

    // Eq. 2: the output symbols are the distinct produced ids, ascending
    tb->out_syms.reserve(tup.size());
    for (const Tuple &t : tup) tb->out_syms.push_back(t.id);
    std::sort(tb->out_syms.begin(), tb->out_syms.end());
    tb->out_syms.erase(std::unique(tb->out_syms.begin(), tb->out_syms.end()), tb->out_syms.end());
    if (tb->out_syms.size() > DOL_MAX_SYMBOLS)
        return fail(DOL_EUNSUPPORTED, "function table produces %zu symbols, more than %d", tb->out_syms.size(),
                    DOL_MAX_SYMBOLS);
    const int32_t S = tb->n_out = static_cast<int32_t>(tb->out_syms.size());

    std::vector<uint32_t> col(tup.size());
    for (size_t t = 0; t < tup.size(); ++t)
        col[t] = static_cast<uint32_t>(std::lower_bound(tb->out_syms.begin(), tb->out_syms.end(), tup[t].id) -
                                       tb->out_syms.begin());

    // counting sorts (stable, so each group keeps ascending (i, j))
    std::vector<uint32_t> col_ptr(S + 1, 0), rowa_ptr(na + 1, 0), rowb_ptr(nb + 1, 0);
    for (size_t t = 0; t < tup.size(); ++t) {
        col_ptr[col[t] + 1]++;
        rowa_ptr[tup[t].i + 1]++;
        rowb_ptr[tup[t].j + 1]++;
    }
    for (int32_t c = 0; c < S; ++c) {
        tb->max_col_len = std::max<int32_t>(tb->max_col_len, static_cast<int32_t>(col_ptr[c + 1]));
        col_ptr[c + 1] += col_ptr[c];
    }
    for (int32_t i = 0; i < na; ++i) rowa_ptr[i + 1] += rowa_ptr[i];
    for (int32_t j = 0; j < nb; ++j) rowb_ptr[j + 1] += rowb_ptr[j];
    std::vector<uint32_t> col_ij(tup.size()), rowa_jc(tup.size()), rowb_ic(tup.size());
    std::vector<uint32_t> rowb_pos(S == na ? tup.size() : 0);
    {
        std::vector<uint32_t> fc(col_ptr.begin(), col_ptr.end() - 1), fa(rowa_ptr.begin(), rowa_ptr.end() - 1),
            fb(rowb_ptr.begin(), rowb_ptr.end() - 1);
        for (size_t t = 0; t < tup.size(); ++t) {
            const uint32_t i = static_cast<uint32_t>(tup[t].i), j = static_cast<uint32_t>(tup[t].j);
            col_ij[fc[col[t]]++] = pack16(i, j);
            const uint32_t qa = fa[i]++, qb = fb[j]++;
            rowa_jc[qa] = pack16(j, col[t]);
            rowb_ic[qb] = pack16(i, col[t]);
            if (!rowb_pos.empty()) rowb_pos[qb] = qa;
        }
    }
    // sum-like: inside every column i rises by one and j falls by one (f(i,j) depends on i+j only and is injective in it)
    tb->sum_like = !tup.empty();
    for (int32_t c = 0; c < S && tb->sum_like; ++c)
        for (uint32_t q = col_ptr[c] + 1; q < col_ptr[c + 1]; ++q) {
            const uint32_t p0 = col_ij[q - 1], p1 = col_ij[q];
            if ((p1 & 0xffff) != (p0 & 0xffff) + 1 || (p1 >> 16) + 1 != (p0 >> 16)) { tb->sum_like = false; break; }
        }

    tb->conv_like = na > 0 && nb > 0 && tup.size() == static_cast<size_t>(na) * static_cast<size_t>(nb) && S == na + nb - 1;
    for (size_t t = 0; t < tup.size() && tb->conv_like; ++t)
        tb->conv_like = col[t] == static_cast<uint32_t>(tup[t].i + tup[t].j);

    std::vector<uint32_t> long_rows;
    for (int32_t i = 0; i < na; ++i) {
        if (rowa_ptr[i + 1] - rowa_ptr[i] > static_cast<uint32_t>(kLongTableRow)) { long_rows.push_back(static_cast<uint32_t>(i)); ++tb->n_long_rowa; }
        tb->max_rowa_len = std::max(tb->max_rowa_len, static_cast<int32_t>(rowa_ptr[i + 1] - rowa_ptr[i]));
    }
    for (int32_t j = 0; j < nb; ++j)
        if (rowb_ptr[j + 1] - rowb_ptr[j] > static_cast<uint32_t>(kLongTableRow)) long_rows.push_back(static_cast<uint32_t>(na + j));

    // long columns: the huge ones first, then those above `wave_above`, then the rest
    auto long_list = [&](uint32_t longer_than, uint32_t wave_above, uint32_t huge_above, int32_t *n_huge, int32_t *n_wave) {
        std::vector<uint32_t> huge, wave, rest;
        for (int32_t c = 0; c < S; ++c) {
            const uint32_t len = col_ptr[c + 1] - col_ptr[c];
            if (len > huge_above) huge.push_back(static_cast<uint32_t>(c));
            else if (len > wave_above) wave.push_back(static_cast<uint32_t>(c));
            else if (len > longer_than) rest.push_back(static_cast<uint32_t>(c));
        }
        *n_huge = static_cast<int32_t>(huge.size());
        *n_wave = static_cast<int32_t>(wave.size());
        huge.insert(huge.end(), wave.begin(), wave.end());
        huge.insert(huge.end(), rest.begin(), rest.end());
        return huge;
    };
    int32_t unused = 0;
    const std::vector<uint32_t> long_cols = long_list(kLongTableCol, kLongTableCol, kHugeTableCol, &tb->n_huge_cols, &unused);
    const std::vector<uint32_t> dtkp_long_cols =
        long_list(kLongDtkpCol, kWaveDtkpCol, kHugeDtkpCol, &tb->n_huge_dtkp_cols, &tb->n_wave_dtkp_cols);

    if (hipGetDevice(&tb->device) != hipSuccess) tb->device = 0;
    hipError_t e;
    if ((e = tb->long_rows.upload(long_rows)) != hipSuccess) return hip_fail(e, "uploading the function table");
    const std::vector<uint32_t> col_order = columns_by_length(col_ptr, S, kLongDtkpCol);
    if ((e = tb->long_cols.upload(long_cols)) != hipSuccess || (e = tb->dtkp_long_cols.upload(dtkp_long_cols)) != hipSuccess ||
        (e = tb->col_order.upload(col_order)) != hipSuccess)
        return hip_fail(e, "uploading the function table");
    std::vector<uint32_t> col_head(static_cast<size_t>(S) * 4, 0xFFFFFFFFu);
    for (int32_t c = 0; c < S; ++c)
        for (uint32_t q = col_ptr[c], u = 0; q < col_ptr[c + 1] && u < 4; ++q, ++u) col_head[static_cast<size_t>(c) * 4 + u] = col_ij[q];
    if ((e = tb->col_head.upload(col_head)) != hipSuccess) return hip_fail(e, "uploading the function table");
    {
        uint32_t longest = 0;
        std::vector<uint32_t> ord_len(static_cast<size_t>(S), 0);
        for (int32_t r = 0; r < S; ++r) {
            const uint32_t len = col_ptr[col_order[r] + 1] - col_ptr[col_order[r]];
            if (len <= static_cast<uint32_t>(kLongDtkpCol)) { ord_len[r] = len; longest = std::max(longest, len); }
        }
        std::vector<uint32_t> ord_tuples(static_cast<size_t>(longest) * S, 0);
        for (int32_t r = 0; r < S; ++r)
            for (uint32_t k = 0; k < ord_len[r]; ++k) ord_tuples[static_cast<size_t>(k) * S + r] = col_ij[col_ptr[col_order[r]] + k];
        if ((e = tb->ord_len.upload(ord_len)) != hipSuccess || (e = tb->ord_tuples.upload(ord_tuples)) != hipSuccess)
            return hip_fail(e, "uploading the function table");
    }
    {
        std::vector<uint32_t> ord(col_head.size());
        for (int32_t r = 0; r < S; ++r)
            for (int u = 0; u < 4; ++u) ord[static_cast<size_t>(r) * 4 + u] = col_head[static_cast<size_t>(col_order[r]) * 4 + u];
        if ((e = tb->col_head_ord.upload(ord)) != hipSuccess) return hip_fail(e, "uploading the function table");
    }
    if ((e = tb->col_ptr.upload(col_ptr)) != hipSuccess || (e = tb->col_ij.upload(col_ij)) != hipSuccess ||
        (e = tb->rowa_ptr.upload(rowa_ptr)) != hipSuccess || (e = tb->rowa_jc.upload(rowa_jc)) != hipSuccess ||
        (e = tb->rowb_ptr.upload(rowb_ptr)) != hipSuccess || (e = tb->rowb_ic.upload(rowb_ic)) != hipSuccess ||
        (e = tb->rowb_pos.upload(rowb_pos)) != hipSuccess)
        return hip_fail(e, "uploading the function table");
    if (!conv_path_ok(tb.get()))
        if (dol_status s2 = lds_plan_build(tb.get(), col_ptr, col_ij, rowa_ptr, rowa_jc, rowb_ptr, rowb_ic)) return s2;
    if (!conv_path_ok(tb.get()) && !tb->lds_fwd_ok && !tb->lds_bwd_ok && nb >= 1 && nb <= kByJMax && na >= 1 &&
        na <= kByJMaxNa && S >= 1 && S <= kByJMaxNa) {
        const int32_t nbp = nb <= 4 ? 4 : nb <= 8 ? 8 : nb <= 10 ? 10 : 16;
        tb->byj_nbp = nbp;
        std::vector<uint16_t> src(static_cast<size_t>(nbp) * S, kByJNone), colof(static_cast<size_t>(nbp) * na, kByJNone);
        std::vector<uint32_t> wave_cols, huge_cols;
        for (int32_t c = 0; c < S; ++c) {
            bool regular = col_ptr[c + 1] - col_ptr[c] <= static_cast<uint32_t>(kLongTableCol);
            for (uint32_t q = col_ptr[c]; q < col_ptr[c + 1] && regular; ++q) {
                uint16_t &slot = src[static_cast<size_t>(col_ij[q] >> 16) * S + c];
                if (slot != kByJNone) regular = false;
                slot = static_cast<uint16_t>(col_ij[q] & 0xffffu);
            }
            if (!regular) {
                const bool is_long = col_ptr[c + 1] - col_ptr[c] > static_cast<uint32_t>(kLongTableCol);
                for (int32_t j = 0; j < nb; ++j) src[static_cast<size_t>(j) * S + c] = kByJNone;
                src[c] = is_long ? kByJWave : kByJList;
                if (is_long) (col_ptr[c + 1] - col_ptr[c] > static_cast<uint32_t>(kHugeTableCol) ? huge_cols : wave_cols).push_back(static_cast<uint32_t>(c));
            }
        }
        tb->n_huge_byj_cols = static_cast<int32_t>(huge_cols.size());
        huge_cols.insert(huge_cols.end(), wave_cols.begin(), wave_cols.end());
        wave_cols.swap(huge_cols);
        for (size_t t = 0; t < tup.size(); ++t) colof[static_cast<size_t>(tup[t].j) * na + tup[t].i] = static_cast<uint16_t>(col[t]);
        if ((e = tb->byj_src.upload(src)) != hipSuccess || (e = tb->byj_col.upload(colof)) != hipSuccess ||
            (e = tb->byj_wave_cols.upload(wave_cols)) != hipSuccess)
            return hip_fail(e, "uploading the function table");
        tb->byj_ok = true;
        tb->byj_fwd = 2 * tup.size() >= static_cast<size_t>(nb) * static_cast<size_t>(S);
    }
    tb->h_col_ptr.swap(col_ptr);
    tb->h_col_ij.swap(col_ij);
    tb->kernel_fwd = damp_kernel_name(tb.get(), false);
    tb->kernel_bwd = damp_kernel_name(tb.get(), true);
    *out = tb.release();
    return DOL_OK;
}

static dol_status check_table_dims(int32_t na, int32_t nb, dol_fn_table **table)
{
    if (!table) return fail(DOL_EINVAL, "table output pointer is NULL");
    *table = nullptr;
    if (na < 0 || nb < 0 || na > DOL_MAX_SYMBOLS || nb > DOL_MAX_SYMBOLS)
        return fail(DOL_ESHAPE, "operand sizes %d x %d outside 0..%d", na, nb, DOL_MAX_SYMBOLS);
    return DOL_OK;
}

// ---------------------------------------------------------------- content-addressed plan caches

static uint64_t fnv1a(const void *data, size_t n, uint64_t h = 1469598103934665603ull)
{
    const unsigned char *p = static_cast<const unsigned char *>(data);
    for (size_t x = 0; x < n; ++x) h = (h ^ p[x]) * 1099511628211ull;
    return h;
}

// At most kCacheMax plans per cache: a program whose predicates or symbol lists keep changing would otherwise grow the
// caches without bound.  Beyond that the plan that has gone unused longest is released (hipFree waits for launches
// that may still read its arrays; plans handed out earlier must not be used after kCacheMax newer ones were made).
constexpr size_t kCacheMax = 4096;

template <typename Plan>
struct Cache {
    struct Entry {
        std::vector<unsigned char> key;
        std::unique_ptr<Plan> plan;
        uint64_t used = 0;
    };
    std::mutex mu;
    std::unordered_multimap<uint64_t, Entry> map;
    uint64_t clock = 0;

    const Plan *find(uint64_t h, const std::vector<unsigned char> &key)
    {
        auto range = map.equal_range(h);
        for (auto it = range.first; it != range.second; ++it)
            if (it->second.key == key) { it->second.used = ++clock; return it->second.plan.get(); }
        return nullptr;
    }
    const Plan *insert(uint64_t h, std::vector<unsigned char> &&key, std::unique_ptr<Plan> &&plan)
    {
        if (map.size() >= kCacheMax) {
            auto oldest = map.begin();
            for (auto it = map.begin(); it != map.end(); ++it)
                if (it->second.used < oldest->second.used) oldest = it;
            map.erase(oldest);
        }
        auto it = map.emplace(h, Entry{std::move(key), std::move(plan), ++clock});
        return it->second.plan.get();
    }
};

static std::vector<unsigned char> make_key(int device, std::initializer_list<std::pair<const void *, size_t>> parts)
{
    std::vector<unsigned char> key(sizeof(int));
    std::memcpy(key.data(), &device, sizeof(int));
    for (const auto &p : parts) {
        const uint64_t n = p.second;
        const unsigned char *nb = reinterpret_cast<const unsigned char *>(&n);
        key.insert(key.end(), nb, nb + sizeof n);
        const unsigned char *d = static_cast<const unsigned char *>(p.first);
        if (n) key.insert(key.end(), d, d + n);
    }
    return key;
}

// (on the heap and never destroyed: no hipFree during static destruction, when the HIP runtime may already be down)
static Cache<FilterPlan> &g_filter_cache = *new Cache<FilterPlan>;
static Cache<UnionPlan> &g_union_cache = *new Cache<UnionPlan>;

dol_status get_filter_plan(int32_t n, const uint8_t *pred, const FilterPlan **plan)
{
    int device = 0;
    (void)hipGetDevice(&device);
    std::vector<uint8_t> norm(static_cast<size_t>(n));
    for (int32_t i = 0; i < n; ++i) norm[i] = pred[i] ? 1 : 0;
    std::vector<unsigned char> key = make_key(device, {{norm.data(), norm.size()}});
    const uint64_t h = fnv1a(key.data(), key.size());
    std::lock_guard<std::mutex> lock(g_filter_cache.mu);
    if ((*plan = g_filter_cache.find(h, key)) != nullptr) return DOL_OK;

    std::unique_ptr<FilterPlan> p(new (std::nothrow) FilterPlan);
    if (!p) return fail(DOL_ENOMEM, "out of host memory");
    p->n_in = n;
    std::vector<int32_t> pos(static_cast<size_t>(n), -1);
    for (int32_t i = 0; i < n; ++i)
        if (norm[i]) {
            pos[i] = static_cast<int32_t>(p->keep_idx.size());
            p->keep_idx.push_back(i);
        }
    p->n_out = static_cast<int32_t>(p->keep_idx.size());
    hipError_t e;
    if ((e = p->d_keep_idx.upload(p->keep_idx)) != hipSuccess || (e = p->d_pos.upload(pos)) != hipSuccess)
        return hip_fail(e, "uploading the filter plan");
    *plan = g_filter_cache.insert(h, std::move(key), std::move(p));
    return DOL_OK;
}

dol_status get_union_plan(int32_t na, const int32_t *sa, int32_t nb, const int32_t *sb, const UnionPlan **plan)
{
    int device = 0;
    (void)hipGetDevice(&device);
    std::vector<unsigned char> key =
        make_key(device, {{sa, sizeof(int32_t) * static_cast<size_t>(na)}, {sb, sizeof(int32_t) * static_cast<size_t>(nb)}});
    const uint64_t h = fnv1a(key.data(), key.size());
    std::lock_guard<std::mutex> lock(g_union_cache.mu);
    if ((*plan = g_union_cache.find(h, key)) != nullptr) return DOL_OK;

    std::unique_ptr<UnionPlan> p(new (std::nothrow) UnionPlan);
    if (!p) return fail(DOL_ENOMEM, "out of host memory");
    p->na = na;
    p->nb = nb;
    std::vector<int32_t> ia, ib, ca(static_cast<size_t>(na)), cb(static_cast<size_t>(nb));
    int32_t i = 0, j = 0;
    while (i < na || j < nb) {            // ascending merge of two ascending id lists
        const int32_t c = static_cast<int32_t>(ia.size());
        if (j >= nb || (i < na && sa[i] < sb[j])) {
            p->out_syms.push_back(sa[i]); ia.push_back(i); ib.push_back(-1); ca[i++] = c;
        } else if (i >= na || sb[j] < sa[i]) {
            p->out_syms.push_back(sb[j]); ia.push_back(-1); ib.push_back(j); cb[j++] = c;
        } else {
            p->out_syms.push_back(sa[i]); ia.push_back(i); ib.push_back(j); ca[i++] = c; cb[j++] = c;
        }
    }
    p->n_out = static_cast<int32_t>(ia.size());
    hipError_t e;
    if ((e = p->d_ia.upload(ia)) != hipSuccess || (e = p->d_ib.upload(ib)) != hipSuccess ||
        (e = p->d_ca.upload(ca)) != hipSuccess || (e = p->d_cb.upload(cb)) != hipSuccess)
        return hip_fail(e, "uploading the union plan");
    *plan = g_union_cache.insert(h, std::move(key), std::move(p));
    return DOL_OK;
}

static Cache<UnionPlan> &g_filter_union_cache = *new Cache<UnionPlan>;

// union(filter(d, pred), c) as ONE merge plan over the unfiltered operand: ia[u] is a position in d (of a kept
// symbol) or -1, ca[x] is the output column of d's symbol x or -1 when the predicate drops it.
dol_status get_filter_union_plan(int32_t n, const int32_t *sd, const uint8_t *pred, int32_t nc, const int32_t *sc,
                                 const UnionPlan **plan)
{
    int device = 0;
    (void)hipGetDevice(&device);
    std::vector<uint8_t> norm(static_cast<size_t>(n));
    for (int32_t i = 0; i < n; ++i) norm[i] = pred[i] ? 1 : 0;
    std::vector<unsigned char> key = make_key(device, {{norm.data(), norm.size()},
                                                       {sd, sizeof(int32_t) * static_cast<size_t>(n)},
                                                       {sc, sizeof(int32_t) * static_cast<size_t>(nc)}});
    const uint64_t h = fnv1a(key.data(), key.size());
    std::lock_guard<std::mutex> lock(g_filter_union_cache.mu);
    if ((*plan = g_filter_union_cache.find(h, key)) != nullptr) return DOL_OK;

    std::unique_ptr<UnionPlan> p(new (std::nothrow) UnionPlan);
    if (!p) return fail(DOL_ENOMEM, "out of host memory");
    p->na = n;
    p->nb = nc;
    std::vector<int32_t> ia, ib, ca(static_cast<size_t>(n), -1), cb(static_cast<size_t>(nc));
    int32_t i = 0, j = 0;
    while (true) {                          // ascending merge of the kept ids of d with the ids of c
        while (i < n && !norm[i]) ++i;
        if (i >= n && j >= nc) break;
        const int32_t col = static_cast<int32_t>(ia.size());
        if (j >= nc || (i < n && sd[i] < sc[j])) {
            p->out_syms.push_back(sd[i]); ia.push_back(i); ib.push_back(-1); ca[i++] = col;
        } else if (i >= n || sc[j] < sd[i]) {
            p->out_syms.push_back(sc[j]); ia.push_back(-1); ib.push_back(j); cb[j++] = col;
        } else {
            p->out_syms.push_back(sd[i]); ia.push_back(i); ib.push_back(j); ca[i++] = col; cb[j++] = col;
        }
    }
    p->n_out = static_cast<int32_t>(ia.size());
    p->aligned = p->n_out == nc && n <= nc;
    for (int32_t c = 0; c < p->n_out && p->aligned; ++c) p->aligned = ib[c] == c && (ia[c] == c || ia[c] < 0);
    hipError_t e;
    if ((e = p->d_ia.upload(ia)) != hipSuccess || (e = p->d_ib.upload(ib)) != hipSuccess ||
        (e = p->d_ca.upload(ca)) != hipSuccess || (e = p->d_cb.upload(cb)) != hipSuccess)
        return hip_fail(e, "uploading the filter-union plan");
    *plan = g_filter_union_cache.insert(h, std::move(key), std::move(p));
    return DOL_OK;
}

struct I32Array {
    DevArray<int32_t> d;
};
static Cache<I32Array> &g_i32_cache = *new Cache<I32Array>;

// Device copy of a small host int32 array, cached by content.
dol_status get_i32_array(int32_t n, const int32_t *data, const int32_t **dptr)
{
    int device = 0;
    (void)hipGetDevice(&device);
    std::vector<unsigned char> key = make_key(device, {{data, sizeof(int32_t) * static_cast<size_t>(n)}});
    const uint64_t h = fnv1a(key.data(), key.size());
    std::lock_guard<std::mutex> lock(g_i32_cache.mu);
    const I32Array *hit = g_i32_cache.find(h, key);
    if (!hit) {
        std::unique_ptr<I32Array> p(new (std::nothrow) I32Array);
        if (!p) return fail(DOL_ENOMEM, "out of host memory");
        hipError_t e = p->d.upload(std::vector<int32_t>(data, data + n));
        if (e != hipSuccess) return hip_fail(e, "uploading an index array");
        hit = g_i32_cache.insert(h, std::move(key), std::move(p));
    }
    *dptr = hit->d.ptr;
    return DOL_OK;
}

dol_status make_group_masks(const dol_prov *prov, GroupMasks *gm)
{
    gm->n = 0;
    if (!prov->fact_group) return DOL_OK;
    std::unordered_map<int32_t, uint64_t> by_group;
    for (int32_t f = 0; f < prov->n_facts; ++f) {
        if (prov->fact_group[f] < 0) return fail(DOL_EINVAL, "fact_group[%d] is negative", f);
        by_group[prov->fact_group[f]] |= uint64_t(1) << f;
    }
    std::vector<uint64_t> masks;
    for (const auto &kv : by_group)
        if (__builtin_popcountll(kv.second) >= 2) masks.push_back(kv.second);
    std::sort(masks.begin(), masks.end());
    if (masks.size() > 32) return fail(DOL_EUNSUPPORTED, "more than 32 exclusion groups with two or more facts");
    gm->n = static_cast<int32_t>(masks.size());
    for (size_t x = 0; x < masks.size(); ++x) gm->m[x] = masks[x];
    return DOL_OK;
}

}  // namespace dol

// ---------------------------------------------------------------- C ABI: tables and plans

extern "C" {

dol_status dol_fn_table_create_dense(int32_t na, int32_t nb, const int32_t *out_id, dol_fn_table **table)
{
    if (dol_status st = dol::check_table_dims(na, nb, table)) return st;
    if (!out_id && na > 0 && nb > 0) return dol::fail(DOL_EINVAL, "out_id is NULL");
    std::vector<dol::Tuple> tup;
    tup.reserve(static_cast<size_t>(na) * static_cast<size_t>(nb));
    for (int32_t i = 0; i < na; ++i)
        for (int32_t j = 0; j < nb; ++j) {
            const int32_t id = out_id[static_cast<size_t>(i) * nb + j];
            if (id < -1) return dol::fail(DOL_EINVAL, "out_id[%d,%d] = %d; ids are >= 0 or -1 for a rejected tuple", i, j, id);
            if (id >= 0) tup.push_back({i, j, id});
        }
    return dol::build_table(na, nb, tup, table);
}

dol_status dol_fn_table_create_if(int32_t na, int32_t nb, const int32_t *out_id, const uint8_t *cond,
                                  dol_fn_table **table)
{
    if (dol_status st = dol::check_table_dims(na, nb, table)) return st;
    if ((!out_id || !cond) && na > 0 && nb > 0) return dol::fail(DOL_EINVAL, "out_id or cond is NULL");
    std::vector<dol::Tuple> tup;
    for (int32_t i = 0; i < na; ++i)
        for (int32_t j = 0; j < nb; ++j) {
            const size_t e = static_cast<size_t>(i) * nb + j;
            if (!cond[e]) continue;
            if (out_id[e] < 0) return dol::fail(DOL_EINVAL, "out_id[%d,%d] = %d is negative where the condition holds", i, j, out_id[e]);
            tup.push_back({i, j, out_id[e]});
        }
    return dol::build_table(na, nb, tup, table);
}

dol_status dol_fn_table_create_sparse(int32_t na, int32_t nb, int64_t n, const int32_t *i, const int32_t *j,
                                      const int32_t *out_id, dol_fn_table **table)
{
    if (dol_status st = dol::check_table_dims(na, nb, table)) return st;
    if (n < 0) return dol::fail(DOL_EINVAL, "negative tuple count");
    if (n > 0 && (!i || !j || !out_id)) return dol::fail(DOL_EINVAL, "tuple arrays are NULL");
    std::vector<dol::Tuple> tup;
    tup.reserve(static_cast<size_t>(n));
    for (int64_t t = 0; t < n; ++t) {
        if (i[t] < 0 || i[t] >= na || j[t] < 0 || j[t] >= nb)
            return dol::fail(DOL_ESHAPE, "tuple %lld = (%d, %d) outside %d x %d", static_cast<long long>(t), i[t], j[t], na, nb);
        if (out_id[t] < 0) return dol::fail(DOL_EINVAL, "tuple %lld produces the negative id %d", static_cast<long long>(t), out_id[t]);
        tup.push_back({i[t], j[t], out_id[t]});
    }
    return dol::build_table(na, nb, tup, table);
}

int32_t dol_fn_table_n_out(const dol_fn_table *table) { return table ? table->n_out : 0; }

const int32_t *dol_fn_table_out_syms(const dol_fn_table *table) { return table ? table->out_syms.data() : nullptr; }

void dol_fn_table_destroy(dol_fn_table *table) { delete table; }

const char *dol_fn_table_kernel(const dol_fn_table *table, int32_t which)
{
    if (!table) return "";
    return which ? table->kernel_bwd.c_str() : table->kernel_fwd.c_str();
}

const char *dol_fn_table_kernel_at(const dol_fn_table *table, int32_t which, int64_t batch)
{
    static thread_local std::string name;
    if (!table) return "";
    name = dol::damp_kernel_name(table, which != 0, batch);
    return name.c_str();
}

dol_status dol_filter_plan(const dol_dist *d, const uint8_t *pred_mask, int32_t *n_out, int32_t *out_syms)
{
    if (!d || !n_out) return dol::fail(DOL_EINVAL, "NULL argument");
    if (d->n_sym < 0 || d->n_sym > DOL_MAX_SYMBOLS) return dol::fail(DOL_ESHAPE, "n_sym %d outside 0..%d", d->n_sym, DOL_MAX_SYMBOLS);
    if (d->n_sym > 0 && (!pred_mask || (out_syms && !d->sym_ids))) return dol::fail(DOL_EINVAL, "pred_mask or sym_ids is NULL");
    int32_t m = 0;
    for (int32_t i = 0; i < d->n_sym; ++i)
        if (pred_mask[i]) {
            if (out_syms) out_syms[m] = d->sym_ids[i];
            ++m;
        }
    *n_out = m;
    return DOL_OK;
}

dol_status dol_filter_union_plan(const dol_dist *d, const uint8_t *pred_mask, const dol_dist *c, int32_t *n_out,
                                 int32_t *out_syms)
{
    if (!d || !c || !n_out || !pred_mask) return dol::fail(DOL_EINVAL, "NULL argument");
    if (d->n_sym < 0 || c->n_sym < 0 || d->n_sym > DOL_MAX_SYMBOLS || c->n_sym > DOL_MAX_SYMBOLS)
        return dol::fail(DOL_ESHAPE, "n_sym outside 0..%d", DOL_MAX_SYMBOLS);
    if ((d->n_sym > 0 && !d->sym_ids) || (c->n_sym > 0 && !c->sym_ids)) return dol::fail(DOL_EINVAL, "sym_ids is NULL");
    for (int32_t i = 1; i < d->n_sym; ++i)
        if (d->sym_ids[i - 1] >= d->sym_ids[i]) return dol::fail(DOL_EINVAL, "d.sym_ids not strictly ascending at %d", i);
    for (int32_t j = 1; j < c->n_sym; ++j)
        if (c->sym_ids[j - 1] >= c->sym_ids[j]) return dol::fail(DOL_EINVAL, "c.sym_ids not strictly ascending at %d", j);
    int32_t i = 0, j = 0, m = 0;
    while (true) {
        while (i < d->n_sym && !pred_mask[i]) ++i;
        if (i >= d->n_sym && j >= c->n_sym) break;
        int32_t id;
        if (j >= c->n_sym || (i < d->n_sym && d->sym_ids[i] < c->sym_ids[j])) id = d->sym_ids[i++];
        else if (i >= d->n_sym || c->sym_ids[j] < d->sym_ids[i]) id = c->sym_ids[j++];
        else { id = d->sym_ids[i++]; ++j; }
        if (out_syms) out_syms[m] = id;
        ++m;
    }
    *n_out = m;
    return DOL_OK;
}

dol_status dol_union_plan(const dol_dist *a, const dol_dist *b, int32_t *n_out, int32_t *out_syms)
{
    if (!a || !b || !n_out) return dol::fail(DOL_EINVAL, "NULL argument");
    if (a->n_sym < 0 || b->n_sym < 0 || a->n_sym > DOL_MAX_SYMBOLS || b->n_sym > DOL_MAX_SYMBOLS)
        return dol::fail(DOL_ESHAPE, "n_sym outside 0..%d", DOL_MAX_SYMBOLS);
    if ((a->n_sym > 0 && !a->sym_ids) || (b->n_sym > 0 && !b->sym_ids)) return dol::fail(DOL_EINVAL, "sym_ids is NULL");
    for (int32_t i = 1; i < a->n_sym; ++i)
        if (a->sym_ids[i - 1] >= a->sym_ids[i]) return dol::fail(DOL_EINVAL, "a.sym_ids not strictly ascending at %d", i);
    for (int32_t j = 1; j < b->n_sym; ++j)
        if (b->sym_ids[j - 1] >= b->sym_ids[j]) return dol::fail(DOL_EINVAL, "b.sym_ids not strictly ascending at %d", j);
    int32_t i = 0, j = 0, m = 0;
    while (i < a->n_sym || j < b->n_sym) {
        int32_t id;
        if (j >= b->n_sym || (i < a->n_sym && a->sym_ids[i] < b->sym_ids[j])) id = a->sym_ids[i++];
        else if (i >= a->n_sym || b->sym_ids[j] < a->sym_ids[i]) id = b->sym_ids[j++];
        else { id = a->sym_ids[i++]; ++j; }
        if (out_syms) out_syms[m] = id;
        ++m;
    }
    *n_out = m;
    return DOL_OK;
}

const char *dol_last_error(void) { return dol::g_last_error.c_str(); }

const char *dol_version(void) { return "0.1.0"; }

}  // extern "C"
