// Cache of compiled code objects.
//
// A trial compiles the template under configuration x, runs it and times it (Sec. 3); the compile
// is by far the longest of the three.  Runs of Alg. 1 that differ only in the seed, or sweeps over
// q and lambda, revisit many configurations, and so does a repeated tuning job in a new process.
// The cache maps (template text, constants, compile options) to the gfx950 code object: in memory
// (bounded, oldest entries dropped first) and, when a directory is configured, in one file per
// entry, written under a temporary name and renamed so that readers never see half a file.
#include "code_cache.hpp"

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <list>
#include <memory>
#include <mutex>
#include <unordered_map>

#include <sys/stat.h>
#include <unistd.h>

#include "common.hpp"

namespace opevo {

const char *template_source(const char *name);
const char *compile_options_tag();

namespace {

struct Entry {
    std::string key;
    std::shared_ptr<const std::vector<char>> code;
};

std::mutex g_mu;
std::list<Entry> g_order;   // oldest first
std::unordered_map<std::string, std::list<Entry>::iterator> g_map;
int64_t g_mem_bytes = 0;
int64_t g_mem_cap = int64_t(256) << 20;
std::string g_dir;
bool g_env_read = false;
int64_t g_hits = 0, g_disk_hits = 0, g_misses = 0;

const char kMagic[8] = {'O', 'P', 'E', 'V', 'O', 'C', 'O', '1'};

uint64_t fnv1a(const std::string &s, uint64_t h)
{
    for (unsigned char c : s) {
        h ^= c;
        h *= 0x100000001B3ull;
    }
    return h;
}

void read_env_locked()
{
    if (g_env_read) return;
    g_env_read = true;
    if (const char *d = getenv("OPEVO_CODE_CACHE_DIR"))
        if (*d && g_dir.empty()) g_dir = d;
}

std::string file_of(const std::string &key)
{
    char name[48];
    snprintf(name, sizeof name, "/%016llx%016llx.co", (unsigned long long)fnv1a(key, 0xCBF29CE484222325ull),
             (unsigned long long)fnv1a(key, 0x84222325CBF29CE4ull));
    return g_dir + name;
}

void insert_locked(const std::string &key, std::shared_ptr<const std::vector<char>> code)
{
    if (g_mem_cap <= 0 || int64_t(code->size()) > g_mem_cap) return;
    auto it = g_map.find(key);
    if (it != g_map.end()) return;
    g_order.push_back(Entry{key, code});
    g_map[key] = std::prev(g_order.end());
    g_mem_bytes += int64_t(code->size());
    while (g_mem_bytes > g_mem_cap && !g_order.empty()) {
        g_mem_bytes -= int64_t(g_order.front().code->size());
        g_map.erase(g_order.front().key);
        g_order.pop_front();
    }
}

bool read_file(const std::string &path, const std::string &key, std::vector<char> &code)
{
    FILE *f = fopen(path.c_str(), "rb");
    if (!f) return false;
    bool ok = false;
    char magic[8];
    uint64_t klen = 0, clen = 0;
    std::string k;
    if (fread(magic, 1, 8, f) == 8 && !memcmp(magic, kMagic, 8) && fread(&klen, 8, 1, f) == 1 &&
        klen == key.size()) {
        k.resize(klen);
        if ((klen == 0 || fread(&k[0], 1, klen, f) == klen) && k == key && fread(&clen, 8, 1, f) == 1 &&
            clen > 0 && clen < (uint64_t(1) << 30)) {
            code.resize(clen);
            // the length is checked against the file: one byte past the code must be the end
            char extra;
            ok = fread(code.data(), 1, clen, f) == clen && fread(&extra, 1, 1, f) == 0;
        }
    }
    fclose(f);
    if (!ok) code.clear();
    return ok;
}

void write_file(const std::string &path, const std::string &key, const std::vector<char> &code)
{
    static int counter = 0;
    char suffix[64];
    snprintf(suffix, sizeof suffix, ".tmp.%d.%d", int(getpid()), counter++);
    const std::string tmp = path + suffix;
    FILE *f = fopen(tmp.c_str(), "wb");
    if (!f) return;
    const uint64_t klen = key.size(), clen = code.size();
    const bool ok = fwrite(kMagic, 1, 8, f) == 8 && fwrite(&klen, 8, 1, f) == 1 &&
                    fwrite(key.data(), 1, klen, f) == klen && fwrite(&clen, 8, 1, f) == 1 &&
                    fwrite(code.data(), 1, clen, f) == clen;
    const bool closed = fclose(f) == 0;
    if (!ok || !closed || rename(tmp.c_str(), path.c_str()) != 0) unlink(tmp.c_str());
}

}  // namespace

std::string code_cache_key(const std::string &tmpl, const std::string &defines)
{
    // everything the code object depends on: the two source texts (as hashes), the per-member
    // constants and the fixed compiler options
    const char *prologue = template_source("common");
    const char *body = template_source(tmpl.c_str());
    char hashes[64];
    snprintf(hashes, sizeof hashes, "%016llx.%016llx",
             (unsigned long long)fnv1a(prologue ? prologue : "", 0xCBF29CE484222325ull),
             (unsigned long long)fnv1a(body ? body : "", 0xCBF29CE484222325ull));
    return tmpl + "\n" + hashes + "\n" + compile_options_tag() + "\n" + defines;
}

bool code_cache_get(const std::string &key, std::vector<char> &code)
{
    std::lock_guard<std::mutex> lock(g_mu);
    read_env_locked();
    auto it = g_map.find(key);
    if (it != g_map.end()) {
        code = *it->second->code;
        ++g_hits;
        return true;
    }
    if (!g_dir.empty() && read_file(file_of(key), key, code)) {
        insert_locked(key, std::make_shared<const std::vector<char>>(code));
        ++g_hits;
        ++g_disk_hits;
        return true;
    }
    ++g_misses;
    return false;
}

void code_cache_put(const std::string &key, const std::vector<char> &code)
{
    if (code.empty()) return;
    std::lock_guard<std::mutex> lock(g_mu);
    read_env_locked();
    insert_locked(key, std::make_shared<const std::vector<char>>(code));
    if (!g_dir.empty()) write_file(file_of(key), key, code);
}

int code_cache_configure(const char *dir, int64_t max_memory_bytes)
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_env_read = true;   // an explicit call overrides the environment
    if (dir && *dir) {
        struct stat st;
        if (stat(dir, &st) != 0) {
            if (mkdir(dir, 0777) != 0) return fail(OPEVO_E_ARG, "code_cache_configure: cannot create %s", dir);
        } else if (!S_ISDIR(st.st_mode)) {
            return fail(OPEVO_E_ARG, "code_cache_configure: %s is not a directory", dir);
        }
        if (access(dir, W_OK | X_OK) != 0) return fail(OPEVO_E_ARG, "code_cache_configure: %s is not writable", dir);
        g_dir = dir;
    } else {
        g_dir.clear();
    }
    if (max_memory_bytes >= 0) g_mem_cap = max_memory_bytes;
    while (g_mem_bytes > g_mem_cap && !g_order.empty()) {
        g_mem_bytes -= int64_t(g_order.front().code->size());
        g_map.erase(g_order.front().key);
        g_order.pop_front();
    }
    return OPEVO_OK;
}

void code_cache_clear_memory()
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_order.clear();
    g_map.clear();
    g_mem_bytes = 0;
}

void code_cache_stats(int64_t *hits, int64_t *disk_hits, int64_t *misses, int64_t *entries, int64_t *bytes)
{
    std::lock_guard<std::mutex> lock(g_mu);
    if (hits) *hits = g_hits;
    if (disk_hits) *disk_hits = g_disk_hits;
    if (misses) *misses = g_misses;
    if (entries) *entries = int64_t(g_order.size());
    if (bytes) *bytes = g_mem_bytes;
}

}  // namespace opevo

extern "C" {

int opevo_code_cache_configure(const char *dir, int64_t max_memory_bytes)
{
    return opevo::code_cache_configure(dir, max_memory_bytes);
}

int opevo_code_cache_clear(void)
{
    opevo::code_cache_clear_memory();
    return OPEVO_OK;
}

int opevo_code_cache_stats(int64_t *hits, int64_t *disk_hits, int64_t *misses, int64_t *entries, int64_t *bytes)
{
    opevo::code_cache_stats(hits, disk_hits, misses, entries, bytes);
    return OPEVO_OK;
}

}  // extern "C"
