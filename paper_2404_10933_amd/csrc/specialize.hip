// Specialized form of the lane kernel: estimate_batch.hip compiled at run time
// (hiprtc) with the compiled tables of one set of architecture tables as
// constants, loaded as a module and launched like the built-in kernels.
//
// One build per (device, table words, flavour), made on first use (a fraction of a
// second to a few seconds) and kept until the process ends.  With the environment
// variable LLMEM_KERNEL_CACHE naming a directory, built code objects are also kept
// there and loaded from there by later processes (a file per build, verified
// against the full key and the embedded sources before use).  The sources come from embedded_sources.inc,
// which the build step writes from the files next to this one, so that the
// run-time build and the built-in kernels are the same code.
#include <hip/hip_runtime.h>
#include <hip/hiprtc.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <unistd.h>
#include <string.h>

#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/llmem.h"
#include "estimate_args.h"
#include "embedded_sources.inc"   // EMBEDDED_COUNT, EMBEDDED_NAMES[], EMBEDDED_TEXTS[]; entry 0 is estimate_batch.hip

namespace llmem {

void set_error_text(const char *text);          // estimate.hip: what llmem_strerror(LLMEM_EHIP) returns

namespace {

// waves per SIMD the build aims at: four (128 registers, no spills) for one architecture; with
// several, the code of each sits in a loop over the architectures and needs more registers
inline int specialized_waves(size_t n_arch) { return n_arch == 1 ? 4 : 3; }
const char *const FLAVOUR_KERNEL[3] = {"llmem_specialized_peaks", "llmem_specialized_detail", "llmem_specialized_sweep"};

struct Built {
    // the code object stays in memory as long as the module is loaded: tools that follow code
    // objects (profilers) read it at its original address after the load call has returned
    std::vector<char> *code = nullptr;
    hipModule_t module = nullptr;
    hipFunction_t function = nullptr;
    int per_cu = 1, cu_count = 256;
};

struct Key {
    int device, flavour;
    std::vector<int> first;                     // first word of every architecture
    std::vector<uint32_t> words;
    bool operator<(const Key &o) const
    {
        if (device != o.device) return device < o.device;
        if (flavour != o.flavour) return flavour < o.flavour;
        if (first != o.first) return first < o.first;
        return words < o.words;
    }
};

std::mutex g_lock;
std::map<Key, Built> g_built;                   // never erased: modules stay loaded until the process ends

int fail(const std::string &text)
{
    set_error_text(text.c_str());
    return LLMEM_EHIP;
}

// the words of the compiled tables that the kernel reads: everything up to the end of the last
// architecture's terms
size_t words_used(const EstimateArgs &args)
{
    size_t n = 0;
    for (int q = 0; q < args.n_arch; ++q)
        if ((size_t)args.arch[q].prog_seg[LLMEM_NSEG] > n) n = (size_t)args.arch[q].prog_seg[LLMEM_NSEG];
    return n < (size_t)PROG_WORDS ? n : (size_t)PROG_WORDS;
}

std::string constants_header(const Key &key)
{
    const std::vector<uint32_t> &words = key.words;
    std::string list;
    char item[16];
    for (size_t q = 0; q < words.size(); ++q) {
        snprintf(item, sizeof(item), "0x%08xu,", words[q]);
        list += item;
        if (q % 8 == 7) list += "\n";
    }
    char head[256];
    snprintf(head, sizeof(head), "#pragma once\nnamespace llmem {\nconstexpr int SPEC_WAVES = %d;\nconstexpr int SPEC_N = %zu;\n"
             "constexpr int SPEC_ARCHS = %zu;\n", specialized_waves(key.first.size()), words.size(), key.first.size());
    std::string firsts = "constexpr int SPEC_FIRST[8] = {";
    for (size_t q = 0; q < 8; ++q) firsts += std::to_string(q < key.first.size() ? key.first[q] : 0) + (q < 7 ? ", " : "};\n");
    return std::string(head) + firsts + "__device__ constexpr unsigned SPEC_PROG[SPEC_N] = {\n" + list + "};\n"
           + "__constant__ unsigned SPEC_PROG_MEM[SPEC_N] = {\n" + list + "};\n}\n";
}

// ---- code objects kept between processes (LLMEM_KERNEL_CACHE) ---------------------------------
// File = the identity (architecture name, flavour, waves per SIMD, table words, every embedded
// source), the code object's size and checksum, the code object.  A file whose identity differs
// in any byte, or whose code object is not the one that was written (cut short, altered), is
// ignored and replaced: the loader only ever sees what the compiler produced.
unsigned long long checksum(const char *data, size_t size)
{
    unsigned long long h = 1469598103934665603ull;                       // FNV-1a
    for (size_t q = 0; q < size; ++q) { h ^= (unsigned char)data[q]; h *= 1099511628211ull; }
    return h;
}

std::string identity(const Key &key, const char *arch_name)
{
    std::string id = std::string("llmem-specialized-2|") + arch_name + "|" + std::to_string(key.flavour) + "|"
                     + std::to_string(specialized_waves(key.first.size())) + "|";
    for (int f : key.first) id += std::to_string(f) + ",";
    id += "|";
    id.append(reinterpret_cast<const char *>(key.words.data()), key.words.size() * sizeof(uint32_t));
    for (int q = 0; q < EMBEDDED_COUNT; ++q) { id += "|"; id += EMBEDDED_TEXTS[q]; }
    return id;
}

std::string cache_path(const std::string &id)
{
    const char *dir = getenv("LLMEM_KERNEL_CACHE");
    if (!dir || !dir[0]) return std::string();
    unsigned long long h = 1469598103934665603ull;                       // FNV-1a: the file's name only
    for (unsigned char c : id) { h ^= c; h *= 1099511628211ull; }
    char name[64];
    snprintf(name, sizeof(name), "/llmem-%016llx.co", h);
    return std::string(dir) + name;
}

bool cache_read(const std::string &path, const std::string &id, std::vector<char> *code)
{
    FILE *f = fopen(path.c_str(), "rb");
    if (!f) return false;
    std::vector<char> all;
    char chunk[65536];
    size_t got;
    while ((got = fread(chunk, 1, sizeof(chunk), f)) > 0) all.insert(all.end(), chunk, chunk + got);
    fclose(f);
    unsigned long long id_size = 0, code_size = 0, code_sum = 0;
    if (all.size() < sizeof(id_size)) return false;
    memcpy(&id_size, all.data(), sizeof(id_size));
    const size_t head = sizeof(id_size) + id.size() + sizeof(code_size) + sizeof(code_sum);
    if (id_size != id.size() || all.size() <= head) return false;
    if (memcmp(all.data() + sizeof(id_size), id.data(), id.size()) != 0) return false;
    memcpy(&code_size, all.data() + sizeof(id_size) + id.size(), sizeof(code_size));
    memcpy(&code_sum, all.data() + sizeof(id_size) + id.size() + sizeof(code_size), sizeof(code_sum));
    if (code_size != all.size() - head || checksum(all.data() + head, all.size() - head) != code_sum) return false;
    code->assign(all.begin() + head, all.end());
    return true;
}

void cache_write(const std::string &path, const std::string &id, const std::vector<char> &code)
{
    const std::string tmp = path + ".tmp" + std::to_string((long long)getpid());
    FILE *f = fopen(tmp.c_str(), "wb");
    if (!f) return;                                                    // an unwritable cache is no error
    const unsigned long long id_size = id.size(), code_size = code.size(), code_sum = checksum(code.data(), code.size());
    const bool ok = fwrite(&id_size, sizeof(id_size), 1, f) == 1 && fwrite(id.data(), 1, id.size(), f) == id.size()
                    && fwrite(&code_size, sizeof(code_size), 1, f) == 1 && fwrite(&code_sum, sizeof(code_sum), 1, f) == 1
                    && fwrite(code.data(), 1, code.size(), f) == code.size();
    if (fclose(f) != 0 || !ok || rename(tmp.c_str(), path.c_str()) != 0) remove(tmp.c_str());
}

int compile(const Key &key, const char *arch_name, std::vector<char> *code);

int build(const Key &key, Built *out)
{
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, key.device) != hipSuccess) return fail("no device properties");
    const std::string id = identity(key, prop.gcnArchName);
    const std::string path = cache_path(id);
    out->code = new std::vector<char>();
    out->cu_count = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    std::string problem;
    for (int attempt = 0; attempt < 2; ++attempt) {
        // first a kept code object, if there is one; a kept one that does not load is built again
        const bool kept = attempt == 0 && !path.empty() && cache_read(path, id, out->code);
        if (!kept) {
            const int rc = compile(key, prop.gcnArchName, out->code);
            if (rc != LLMEM_OK) { delete out->code; out->code = nullptr; return rc; }
            if (!path.empty()) cache_write(path, id, *out->code);
        }
        hipError_t e;
        try {
            e = hipModuleLoadData(&out->module, out->code->data());
        } catch (...) {                          // the loader's own C++ errors must not cross the C boundary
            e = hipErrorInvalidImage;
        }
        if (e == hipSuccess) {
            e = hipModuleGetFunction(&out->function, out->module, FLAVOUR_KERNEL[key.flavour]);
            if (e == hipSuccess) return LLMEM_OK;
            (void)hipModuleUnload(out->module);
            out->module = nullptr;
        }
        problem = std::string("loading the specialized kernel: ") + hipGetErrorString(e);
        (void)hipGetLastError();
        if (!kept) break;
    }
    delete out->code;
    out->code = nullptr;
    return fail(problem);
}

int compile(const Key &key, const char *arch_name, std::vector<char> *code)
{
    const std::string constants = constants_header(key);
    std::vector<const char *> names, texts;
    for (int q = 1; q < EMBEDDED_COUNT; ++q) { names.push_back(EMBEDDED_NAMES[q]); texts.push_back(EMBEDDED_TEXTS[q]); }
    names.push_back("specialized_prog.h");
    texts.push_back(constants.c_str());
    hiprtcProgram program;
    if (hiprtcCreateProgram(&program, EMBEDDED_TEXTS[0], EMBEDDED_NAMES[0], (int)names.size(), texts.data(), names.data())
        != HIPRTC_SUCCESS)
        return fail("run-time compiler: cannot create the program");
    const std::string arch = std::string("--offload-arch=") + arch_name;
    const std::string entry = std::string("-DLLMEM_SPEC_FLAVOUR=") + std::to_string(key.flavour);
    const char *options[] = {arch.c_str(), "-O3", "-std=c++17", "-DLLMEM_SPECIALIZED", entry.c_str(),
                             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
    const hiprtcResult compiled = hiprtcCompileProgram(program, (int)(sizeof(options) / sizeof(options[0])), options);
    if (compiled != HIPRTC_SUCCESS) {
        size_t size = 0;
        std::string log;
        if (hiprtcGetProgramLogSize(program, &size) == HIPRTC_SUCCESS && size > 1) {
            log.resize(size);
            hiprtcGetProgramLog(program, &log[0]);
        }
        hiprtcDestroyProgram(&program);
        return fail("run-time compiler: " + std::string(hiprtcGetErrorString(compiled)) + ": " + log.substr(0, 160));
    }
    size_t code_size = 0;
    hiprtcGetCodeSize(program, &code_size);
    code->resize(code_size);
    hiprtcGetCode(program, code->data());
    hiprtcDestroyProgram(&program);
    return LLMEM_OK;
}

}  // namespace

int launch_specialized(const EstimateArgs &args, int flavour, long long n_batch, hipStream_t stream)
{
    if (flavour < 0 || flavour > 2 || !args.use_program || args.n_arch < 1 || args.n_arch > LLMEM_MAX_ARCH)
        return LLMEM_EINVAL_TABLE;
    Key key;
    if (hipGetDevice(&key.device) != hipSuccess) return fail("no current device");
    key.flavour = flavour;
    for (int q = 0; q < args.n_arch; ++q) key.first.push_back(args.arch[q].prog_first);
    key.words.assign(args.prog, args.prog + words_used(args));
    const size_t lds_bytes = batch_kernel_lds_bytes(args);
    Built built;
    {
        std::lock_guard<std::mutex> hold(g_lock);
        auto at = g_built.find(key);
        if (at == g_built.end()) {
            const int rc = build(key, &built);
            if (rc != LLMEM_OK) return rc;
            int per_cu = 0;
            if (hipModuleOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, built.function, 64 * BATCH_WAVES, lds_bytes)
                    == hipSuccess && per_cu > 0)
                built.per_cu = per_cu;
            at = g_built.emplace(key, built).first;
        }
        built = at->second;
    }
    long long blocks = (n_batch + BATCH_WAVES - 1) / BATCH_WAVES;
    const long long resident = (long long)built.per_cu * built.cu_count * 16;   // as for the built-in compiled form
    if (blocks > resident) blocks = resident;
    EstimateArgs copy = args;
    void *params[] = {&copy};
    const hipError_t e = hipModuleLaunchKernel(built.function, (unsigned)blocks, 1, 1, 64 * BATCH_WAVES, 1, 1,
                                               (unsigned)lds_bytes, stream, params, nullptr);
    if (e != hipSuccess) return fail(std::string("launching the specialized kernel: ") + hipGetErrorString(e));
    return LLMEM_OK;
}

}  // namespace llmem
