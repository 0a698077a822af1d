// Run-time compilation of generated kernels for gfx950 and the in-process code cache
// (paper section 2.2.3: generated code is compiled when needed and cached so that identical
// code is never compiled twice; here the key is the generated source itself).
#include <hip/hip_runtime.h>
#include <hip/hiprtc.h>

#include <unistd.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <condition_variable>
#include <mutex>
#include <unordered_map>
#include <unordered_set>

#include "ewf_internal.h"

namespace ewf {

static const char kPrelude[] =
#include "ewf_prelude_embed.inc"
    ;

const char *prelude_source() { return kPrelude; }

namespace {
std::mutex g_mutex;
std::string g_cache_dir;                                                    // empty: no disk cache
int g_stat_mem_hits = 0, g_stat_disk_hits = 0, g_stat_compiles = 0;

// FNV-1a with two different offsets: a 128-bit name for a source text
void hash128(const std::string &text, uint64_t out[2])
{
    uint64_t a = 0xcbf29ce484222325ull, b = 0x84222325cbf29ce4ull;
    for (unsigned char ch : text) {
        a = (a ^ ch) * 0x100000001b3ull;
        b = (b ^ (ch + 0x9e)) * 0x100000001b3ull;
    }
    out[0] = a; out[1] = b;
}

std::string disk_name(const std::string &keyed)
{
    uint64_t h[2];
    hash128(keyed, h);
    char buf[64];
    snprintf(buf, sizeof buf, "/ewf_%016llx%016llx.co", (unsigned long long)h[0], (unsigned long long)h[1]);
    return g_cache_dir + buf;
}

// File layout: "EWFC2\n", the length of the keyed source text (8 bytes), that text, the code
// object.  The file name is only a hash of the text; the text itself decides whether the file
// is the one asked for.
bool disk_load(const std::string &keyed, std::vector<char> &code)
{
    FILE *f = fopen(disk_name(keyed).c_str(), "rb");
    if (!f) return false;
    char magic[6];
    uint64_t len = 0;
    bool ok = fread(magic, 1, 6, f) == 6 && memcmp(magic, "EWFC2\n", 6) == 0 && fread(&len, 8, 1, f) == 1 && len == keyed.size();
    if (ok) {
        std::string stored(keyed.size(), '\0');
        ok = fread(&stored[0], 1, stored.size(), f) == stored.size() && stored == keyed;
    }
    if (ok) {
        const long at = ftell(f);
        fseek(f, 0, SEEK_END);
        const long sz = ftell(f) - at;
        fseek(f, at, SEEK_SET);
        ok = at > 0 && sz > 0;
        if (ok) { code.resize((size_t)sz); ok = fread(code.data(), 1, (size_t)sz, f) == (size_t)sz; }
    }
    fclose(f);
    return ok;
}

void disk_store(const std::string &keyed, const std::vector<char> &code)
{
    const std::string name = disk_name(keyed);
    const std::string tmp = name + ".tmp" + std::to_string((long long)getpid());
    FILE *f = fopen(tmp.c_str(), "wb");
    if (!f) return;                                     // an unwritable cache is not an error
    uint64_t len = keyed.size();
    bool ok = fwrite("EWFC2\n", 1, 6, f) == 6 && fwrite(&len, 8, 1, f) == 1 && fwrite(keyed.data(), 1, keyed.size(), f) == keyed.size() &&
              fwrite(code.data(), 1, code.size(), f) == code.size();
    ok = (fclose(f) == 0) && ok;
    if (!ok || rename(tmp.c_str(), name.c_str()) != 0) remove(tmp.c_str());
}
std::unordered_map<std::string, std::vector<char>> g_code;                 // source -> code object
std::unordered_set<std::string> g_in_flight;                               // sources being compiled right now
std::condition_variable g_in_flight_done;
int g_compiling_now = 0, g_compiling_peak = 0;                             // compiler runs in progress, and the most at once
struct Loaded { hipModule_t module; std::unordered_map<std::string, hipFunction_t> fn; };
std::unordered_map<std::string, Loaded> g_loaded;                          // device ordinal + code object bytes -> module
}  // namespace

// The lock covers the tables only.  A source that is being compiled is marked as in flight:
// another thread that wants the same source waits for it, threads with other sources compile at
// the same time.
ewf_status compile_source(const std::string &source, std::vector<char> &code, bool *was_cached)
{
    std::string cache_dir;
    {
        std::unique_lock<std::mutex> lock(g_mutex);
        for (;;) {
            auto it = g_code.find(source);
            if (it != g_code.end()) {
                code = it->second;
                if (was_cached) *was_cached = true;
                g_stat_mem_hits++;
                return EWF_OK;
            }
            if (!g_in_flight.count(source)) break;
            g_in_flight_done.wait(lock);
        }
        g_in_flight.insert(source);
        cache_dir = g_cache_dir;
    }
    if (was_cached) *was_cached = false;
    // whatever happens below, the mark comes off and the waiting threads look again
    struct Unmark {
        const std::string &src;
        ~Unmark()
        {
            std::lock_guard<std::mutex> lock(g_mutex);
            g_in_flight.erase(src);
            g_in_flight_done.notify_all();
        }
    } unmark{source};

    // second level: code objects kept on disk across processes, named by a hash of everything
    // that determines them (device helpers, generated text, compiler options and version)
    std::string keyed;
    if (!cache_dir.empty()) {
        int major = 0, minor = 0;
        hiprtcVersion(&major, &minor);
        keyed = "gfx950 -O3 no-packed-fp32 hiprtc " + std::to_string(major) + "." + std::to_string(minor) + "\n" + kPrelude + "\n" + source;
        if (disk_load(keyed, code)) {
            std::lock_guard<std::mutex> lock(g_mutex);
            g_code.emplace(source, code);
            g_stat_disk_hits++;
            return EWF_OK;
        }
    }
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        g_stat_compiles++;
        g_compiling_now++;
        if (g_compiling_now > g_compiling_peak) g_compiling_peak = g_compiling_now;
    }
    struct Leave { ~Leave() { std::lock_guard<std::mutex> lock(g_mutex); g_compiling_now--; } } leave;
    hiprtcProgram prog;
    const char *hdr_src[] = {kPrelude};
    const char *hdr_name[] = {"ewf_prelude.hip.h"};
    std::string full = "#include \"ewf_prelude.hip.h\"\n" + source;
    hiprtcResult r = hiprtcCreateProgram(&prog, full.c_str(), "ewf_generated.hip", 1, hdr_src, hdr_name);
    if (r != HIPRTC_SUCCESS) { set_error("hiprtcCreateProgram: %s", hiprtcGetErrorString(r)); return EWF_ECOMPILE; }
    // packed-fp32 instructions are switched off for every kernel of this library
    const char *opts[] = {"--offload-arch=gfx950", "-O3", "-std=c++17",
                          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
    r = hiprtcCompileProgram(prog, (int)(sizeof opts / sizeof opts[0]), opts);
    if (r != HIPRTC_SUCCESS) {
        size_t n = 0;
        hiprtcGetProgramLogSize(prog, &n);
        std::string log(n, '\0');
        if (n) hiprtcGetProgramLog(prog, &log[0]);
        hiprtcDestroyProgram(&prog);
        if (getenv("EWF_DUMP_FAILED_SOURCE")) log += "\n---- source ----\n" + full;
        set_error_str("run-time compilation failed: " + log);
        return EWF_ECOMPILE;
    }
    size_t sz = 0;
    hiprtcGetCodeSize(prog, &sz);
    code.resize(sz);
    hiprtcGetCode(prog, code.data());
    hiprtcDestroyProgram(&prog);
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        g_code.emplace(source, code);
    }
    if (!cache_dir.empty()) disk_store(keyed, code);
    return EWF_OK;
}

namespace {
// the environment can name the cache directory before any call is made
struct CacheDirFromEnv {
    CacheDirFromEnv() { const char *d = getenv("EWF_CACHE_DIR"); if (d && *d) g_cache_dir = d; }
} g_cache_dir_from_env;
}  // namespace

void set_cache_dir(const char *path)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    g_cache_dir = path ? path : "";
}

void cache_stats(int *mem_hits, int *disk_hits, int *compiles)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    *mem_hits = g_stat_mem_hits; *disk_hits = g_stat_disk_hits; *compiles = g_stat_compiles;
}

int peak_concurrent_compiles()
{
    std::lock_guard<std::mutex> lock(g_mutex);
    return g_compiling_peak;
}

ewf_status load_function(const std::vector<char> &code, const std::string &entry, void **function, int *device)
{
    int dev = -1;
    hipError_t he = hipGetDevice(&dev);
    if (he != hipSuccess) { set_error("no HIP device: %s", hipGetErrorString(he)); return EWF_EHIP; }
    // (keyed by the code object itself: a hash of it could hand out another expression's kernel)
    std::string key = std::to_string(dev) + ":";
    key.append(code.data(), code.size());
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_loaded.find(key);
    if (it == g_loaded.end()) {
        Loaded l;
        he = hipModuleLoadData(&l.module, code.data());
        if (he != hipSuccess) { set_error("hipModuleLoadData: %s", hipGetErrorString(he)); return EWF_EHIP; }
        it = g_loaded.emplace(key, std::move(l)).first;
    }
    auto f = it->second.fn.find(entry);
    if (f == it->second.fn.end()) {
        hipFunction_t fn;
        he = hipModuleGetFunction(&fn, it->second.module, entry.c_str());
        if (he != hipSuccess) { set_error("hipModuleGetFunction(%s): %s", entry.c_str(), hipGetErrorString(he)); return EWF_EHIP; }
        f = it->second.fn.emplace(entry, fn).first;
    }
    *function = (void *)f->second;
    if (device) *device = dev;
    return EWF_OK;
}

// Largest per-lane scratch (register spill) size, in bytes, that the metadata of a code object
// records for any of its kernels.  The metadata is a MessagePack map; the value follows the
// key ".private_segment_fixed_size" as an unsigned integer.
int64_t code_scratch_bytes(const std::vector<char> &code)
{
    static const char key[] = ".private_segment_fixed_size";
    const size_t klen = sizeof key - 1;
    int64_t worst = 0;
    for (size_t i = 0; i + klen + 1 <= code.size(); i++) {
        if (memcmp(code.data() + i, key, klen) != 0) continue;
        const unsigned char *q = (const unsigned char *)code.data() + i + klen;
        const size_t left = code.size() - (i + klen);
        int64_t v = -1;
        if (left >= 1 && q[0] <= 0x7f) v = q[0];
        else if (left >= 2 && q[0] == 0xcc) v = q[1];
        else if (left >= 3 && q[0] == 0xcd) v = ((int64_t)q[1] << 8) | q[2];
        else if (left >= 5 && q[0] == 0xce) v = ((int64_t)q[1] << 24) | ((int64_t)q[2] << 16) | ((int64_t)q[3] << 8) | q[4];
        if (v > worst) worst = v;
    }
    return worst;
}

// Compute units of the current device; the published MI355X figure when no device is
// present (planning and compiling need none).
int device_cu_count()
{
    static int cached = 0;
    if (cached > 0) return cached;
    int dev = -1, n = 0;
    if (hipGetDevice(&dev) == hipSuccess && dev >= 0 &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) {
        cached = n;
        return n;
    }
    (void)hipGetLastError();
    return 256;
}

}  // namespace ewf
