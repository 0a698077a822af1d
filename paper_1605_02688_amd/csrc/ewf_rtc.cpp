// Run-time compilation of generated kernels for gfx950 and the in-process code cache
// (paper section 2.2.3: generated code is compiled when needed and cached so that identical
// code is never compiled twice; here the key is the generated source itself).
#include <hip/hip_runtime.h>
#include <hip/hiprtc.h>

#include <cstdlib>
#include <cstring>
#include <mutex>
#include <unordered_map>

#include "ewf_internal.h"

namespace ewf {

static const char kPrelude[] =
#include "ewf_prelude_embed.inc"
    ;

const char *prelude_source() { return kPrelude; }

namespace {
std::mutex g_mutex;
std::unordered_map<std::string, std::vector<char>> g_code;                 // source -> code object
struct Loaded { hipModule_t module; std::unordered_map<std::string, hipFunction_t> fn; };
std::unordered_map<std::string, Loaded> g_loaded;                          // device:hash -> module
}  // namespace

ewf_status compile_source(const std::string &source, std::vector<char> &code, bool *was_cached)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_code.find(source);
    if (it != g_code.end()) {
        code = it->second;
        if (was_cached) *was_cached = true;
        return EWF_OK;
    }
    if (was_cached) *was_cached = false;
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
    g_code.emplace(source, code);
    return EWF_OK;
}

ewf_status load_function(const std::vector<char> &code, const std::string &entry, void **function, int *device)
{
    int dev = -1;
    hipError_t he = hipGetDevice(&dev);
    if (he != hipSuccess) { set_error("no HIP device: %s", hipGetErrorString(he)); return EWF_EHIP; }
    std::string key = std::to_string(dev) + ":" + std::to_string(std::hash<std::string>()(std::string(code.data(), code.size()))) +
                      ":" + std::to_string(code.size());
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
