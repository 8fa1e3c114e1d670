// Table of tuned configurations (Section 3.8: the tuner's results are kept and reused).  Host code only: a process-wide
// map from the problem (world size, M, N, K) to what agg_autotune_ag_gemm found best for it, with a text file format so
// that a later process can start from the table instead of tuning again.
#include "agg_internal.h"

#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <tuple>

using namespace agg;

namespace {

typedef std::tuple<int, int, int, int> Key;     // W, M, N, K
std::mutex g_mutex;
std::map<Key, agg_tune_result> g_table;

const char kHeader[] = "agg-tune-table 1";

bool valid_key(int W, int M, int N, int K) { return W >= 1 && W <= kMaxWorld && M >= 0 && N >= 0 && K >= 0; }

bool valid_entry(const agg_tune_result& r)
{
    return r.tile_config >= 0 && r.tile_config < TILE_CONFIGS &&
           (r.tile_order == AGG_ORDER_ROTATED || r.tile_order == AGG_ORDER_SUBCHUNK) && r.producer_workgroups >= 0 &&
           r.producer_workgroups <= 4096 && r.configs_tried >= 0 && r.best_ms >= 0.f;
}

}  // namespace

void agg::tune_table_put(int W, int M, int N, int K, const agg_tune_result& r)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    g_table[Key(W, M, N, K)] = r;
}

extern "C" {

int agg_tune_table_size(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    return (int)g_table.size();
}

int agg_tune_table_clear(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    g_table.clear();
    return AGG_OK;
}

int agg_tune_table_put(int W, int M, int N, int K, const agg_tune_result* r)
{
    if (!r || !valid_key(W, M, N, K) || !valid_entry(*r)) return AGG_ERR_INVALID_ARG;
    tune_table_put(W, M, N, K, *r);
    return AGG_OK;
}

int agg_tune_table_get(int W, int M, int N, int K, agg_tune_result* out)
{
    if (!out) return AGG_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_mutex);
    const auto it = g_table.find(Key(W, M, N, K));
    if (it == g_table.end()) return AGG_ERR_NOT_FOUND;
    *out = it->second;
    return AGG_OK;
}

int agg_tune_table_save(const char* path)
{
    if (!path) return AGG_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_mutex);
    FILE* f = std::fopen(path, "w");
    if (!f) return AGG_ERR_IO;
    bool ok = std::fprintf(f, "%s\n# W M N K tile_config tile_order producer_workgroups configs_tried best_ms\n", kHeader) > 0;
    for (const auto& kv : g_table) {
        const agg_tune_result& r = kv.second;
        ok = ok && std::fprintf(f, "%d %d %d %d %d %d %d %d %.6g\n", std::get<0>(kv.first), std::get<1>(kv.first),
                                std::get<2>(kv.first), std::get<3>(kv.first), r.tile_config, r.tile_order,
                                r.producer_workgroups, r.configs_tried, (double)r.best_ms) > 0;
    }
    ok = (std::fclose(f) == 0) && ok;
    return ok ? AGG_OK : AGG_ERR_IO;
}

int agg_tune_table_load(const char* path)
{
    if (!path) return AGG_ERR_INVALID_ARG;
    FILE* f = std::fopen(path, "r");
    if (!f) return AGG_ERR_IO;
    std::map<Key, agg_tune_result> read;
    char line[256];
    bool header_seen = false, bad = false;
    while (!bad && std::fgets(line, sizeof line, f)) {
        const size_t len = std::strlen(line);
        if (len + 1 == sizeof line && line[len - 1] != '\n') { bad = true; break; }   // a line longer than any this code writes
        char* s = line;
        while (*s == ' ' || *s == '\t') ++s;
        if (*s == '\n' || *s == '\r' || *s == '\0' || *s == '#') continue;
        if (!header_seen) {
            header_seen = std::strncmp(s, kHeader, sizeof kHeader - 1) == 0 &&
                          (s[sizeof kHeader - 1] == '\n' || s[sizeof kHeader - 1] == '\r' || s[sizeof kHeader - 1] == '\0');
            bad = !header_seen;
            continue;
        }
        int W, M, N, K, used = 0;
        agg_tune_result r{};
        double ms = 0.0;
        if (std::sscanf(s, "%d %d %d %d %d %d %d %d %lf %n", &W, &M, &N, &K, &r.tile_config, &r.tile_order,
                        &r.producer_workgroups, &r.configs_tried, &ms, &used) != 9 || s[used] != '\0' ||
            !(ms >= 0.0 && ms < 1e30)) {
            bad = true;
            break;
        }
        r.best_ms = (float)ms;
        if (!valid_key(W, M, N, K) || !valid_entry(r)) { bad = true; break; }
        read[Key(W, M, N, K)] = r;
    }
    const bool io_error = std::ferror(f) != 0;
    std::fclose(f);
    if (io_error) return AGG_ERR_IO;
    if (bad || !header_seen) return AGG_ERR_INVALID_ARG;     // the table in memory is left as it was
    std::lock_guard<std::mutex> lock(g_mutex);
    for (const auto& kv : read) g_table[kv.first] = kv.second;
    return (int)read.size();
}

int agg_tune_table_apply(agg_ctx* c, int M, int N, int K)
{
    if (!c) return AGG_ERR_INVALID_ARG;
    agg_tune_result r;
    const int rc = agg_tune_table_get(c->W, M, N, K, &r);
    if (rc != AGG_OK) return rc;
    c->tile_config = r.tile_config;
    c->tile_order = r.tile_order;
    c->producer_wgs = r.producer_workgroups;
    return AGG_OK;
}

}  // extern "C"
