// Persistent store of search results.  The paper (Section 3) keeps the solutions of earlier
// searches in a local database and returns them without generating or timing anything again;
// here a solution is the launch configuration a timed search selected, kept as one line of
// text per problem in a file the caller names.
//
// Line format (all integers, blank separated):
//   ttc4 gfx950 <dtype> <beta_is_zero> <ndim> <sizes..> <perm..> <stride_a..> <stride_b..> |
//   <kernel_class> <threads> <wg_per_cu> <lds_buffers> <vec_a> <vec_b> <tile x6> <tile_order x6>
//   <digits_a> <dtile_a x4> <dlane_a x4> <digits_b> <dtile_b x4> <dlane_b x4> <row kernel's unroll> | <nt_a> <nt_b> <tile mapping> <microseconds>
// The left part is the key: the fused problem as the planner sees it.  The middle part names a
// candidate by its configuration, not by its rank, so an entry survives changes of the ranking;
// if no candidate of the current library matches, the entry is ignored.  Later lines win.
#include <cstdio>
#include <cstring>
#include <new>
#include <sstream>
#include <string>
#include <vector>

#include "ttc_internal.h"

namespace ttc {

static const char* kMagic = "ttc4";
static const char* kArch = "gfx950";

static std::string problem_key(const Problem& P)
{
    std::ostringstream o;
    o << kMagic << ' ' << kArch << ' ' << P.dtype << ' ' << (P.epilogue == TTC_EPI_AXPBY ? 0 : 1) << ' ' << P.ndim;
    for (int k = 0; k < P.ndim; ++k) o << ' ' << P.size[k];
    for (int k = 0; k < P.ndim; ++k) o << ' ' << P.perm[k];
    for (int k = 0; k < P.ndim; ++k) o << ' ' << P.stride_a[k];
    for (int k = 0; k < P.ndim; ++k) o << ' ' << P.stride_b[k];
    return o.str();
}

static std::vector<long long> config_signature(const Candidate& c)
{
    std::vector<long long> v;
    v.push_back(c.kernel_class); v.push_back(c.threads); v.push_back(c.wg_per_cu);
    v.push_back(c.kp.lds_buffers); v.push_back(c.kp.a.vec); v.push_back(c.kp.b.vec);
    for (int k = 0; k < kMaxDim; ++k) v.push_back(c.tile[k]);
    for (int k = 0; k < kMaxDim; ++k) v.push_back(c.tile_order[k]);
    v.push_back(c.digits_a);
    for (int i = 0; i < kBoxDims; ++i) v.push_back(c.dtile_a[i]);
    for (int i = 0; i < kBoxDims; ++i) v.push_back(c.dlane_a[i]);
    v.push_back(c.digits_b);
    for (int i = 0; i < kBoxDims; ++i) v.push_back(c.dtile_b[i]);
    for (int i = 0; i < kBoxDims; ++i) v.push_back(c.dlane_b[i]);
    v.push_back(c.rows.unroll);
    return v;
}

int cache_store(const ttc_plan_s* plan, const char* path)
{
    const Candidate& c = plan->cands[plan->selected];
    std::ostringstream o;
    o << problem_key(plan->prob) << " |";
    for (long long x : config_signature(c)) o << ' ' << x;
    o << " | " << c.kp.nt_a << ' ' << c.kp.nt_b << ' ' << c.kp.xcd_remap << ' ' << (long long)(c.tuned_ms * 1000.0f + 0.5f) << '\n';
    const std::string line = o.str();
    std::FILE* f = std::fopen(path, "a");
    if (!f) return TTC_ERR_IO;
    const size_t n = std::fwrite(line.data(), 1, line.size(), f);      // one write per entry
    const int rc = std::fclose(f);
    return (n == line.size() && rc == 0) ? TTC_OK : TTC_ERR_IO;
}

int cache_lookup(ttc_plan_s* plan, const char* path)
{
    std::FILE* f = std::fopen(path, "r");
    if (!f) return TTC_ERR_NOT_FOUND;
    const std::string key = problem_key(plan->prob) + " |";
    std::string hit;
    std::vector<char> buf(4096);
    while (std::fgets(buf.data(), (int)buf.size(), f)) {
        if (std::strncmp(buf.data(), key.c_str(), key.size()) == 0) hit.assign(buf.data() + key.size());
    }
    std::fclose(f);
    if (hit.empty()) return TTC_ERR_NOT_FOUND;
    // "<signature> | <nt_a> <nt_b> <tile mapping> <microseconds>"
    std::vector<long long> sig, tailv;
    long long us = 0;
    {
        std::istringstream in(hit);
        std::string tok;
        bool tail = false;
        while (in >> tok) {
            if (tok == "|") { tail = true; continue; }
            char* end = nullptr;
            const long long v = std::strtoll(tok.c_str(), &end, 10);
            if (!end || *end != '\0') return TTC_ERR_NOT_FOUND;          // damaged line: treat as absent
            if (tail) tailv.push_back(v); else sig.push_back(v);
        }
    }
    if (tailv.size() != 4 || (tailv[0] | 1) != 1 || (tailv[1] | 1) != 1 || tailv[2] < 0 || tailv[2] > 10) return TTC_ERR_NOT_FOUND;
    us = tailv[3];
    const int st = complete_plan(plan);           // an entry may name any candidate of the full list
    if (st != TTC_OK) return st;
    for (size_t i = 0; i < plan->cands.size(); ++i) {
        if (config_signature(plan->cands[i]) == sig) {
            // everything is applied to a copy first: a refused entry leaves the plan as it was
            Candidate c = plan->cands[i];
            c.kp.nt_a = (int)tailv[0];
            c.kp.nt_b = (int)tailv[1];
            if (c.kernel_class == TTC_KERNEL_DIRECT && c.kp.nt_a != c.kp.nt_b) return TTC_ERR_NOT_FOUND;   // streams both sides or neither
            if (!set_tile_mapping(&c.kp, (int)tailv[2])) return TTC_ERR_NOT_FOUND;
            c.tuned_ms = (float)us / 1000.0f;
            plan->cands[i] = c;
            plan->selected = (int)i;
            return TTC_OK;
        }
    }
    return TTC_ERR_NOT_FOUND;
}

}  // namespace ttc

extern "C" {

int ttc_plan_cache_store(ttc_plan_t plan, const char* path)
{
    if (!plan || !path) return TTC_ERR_NULL_POINTER;
    try { return ttc::cache_store(plan, path); } catch (const std::bad_alloc&) { return TTC_ERR_ALLOC; } catch (...) { return TTC_ERR_INTERNAL; }
}

int ttc_plan_cache_lookup(ttc_plan_t plan, const char* path)
{
    if (!plan || !path) return TTC_ERR_NULL_POINTER;
    try { return ttc::cache_lookup(plan, path); } catch (const std::bad_alloc&) { return TTC_ERR_ALLOC; } catch (...) { return TTC_ERR_INTERNAL; }
}

}  // extern "C"
