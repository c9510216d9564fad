// Specialized forms of the lane kernel: estimate_batch.hip compiled with the
// compiled tables of one set of architecture tables as constants.
//
// Built ahead of time: the build step compiles one kernel per flavour for every
// table set the library ships with and lists them, with the table words they were
// made from, in aot_registry.inc; a call whose compiled tables equal such a list
// word for word launches that kernel like any built-in one (no compiler, no
// module, nothing allocated).
//
// Built at run time (hiprtc): any other tables, when asked for.  One build per
// (device, table words, flavour), made on first use (a fraction of a second to a
// few seconds) and kept until release_built() or the end of the process.  With the environment variable
// LLMEM_KERNEL_CACHE naming a directory, built code objects are also kept there
// and loaded from there by later processes (a file per build, verified against the
// full key and the embedded sources before use).  The sources come from
// embedded_sources.inc, which the build step writes from the files next to this
// one, so that every form of the kernel is the same code.
#include <hip/hip_runtime.h>
#include <hip/hiprtc.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <unistd.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <map>
#include <memory>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/llmem.h"
#include "estimate_args.h"
#include "embedded_sources.inc"   // EMBEDDED_COUNT, EMBEDDED_NAMES[], EMBEDDED_TEXTS[]; entry 0 is estimate_batch.hip

namespace llmem {
namespace {
// a kernel built into the library and the compiled tables it was made from
struct Prebuilt {
    const char *name;
    int flavour, n_arch;
    int first[LLMEM_MAX_ARCH];
    int n_words;
    const uint32_t *words;
    const void *(*entry)();                     // the kernel, as the launch calls take it
};
}  // namespace
}  // namespace llmem
#ifndef LLMEM_AOT_REGISTRY
#define LLMEM_AOT_REGISTRY "aot_registry.inc"
#endif
#include LLMEM_AOT_REGISTRY       // PREBUILT[], PREBUILT_COUNT (written by the build step; an empty list
                                  // while the build step is still making the kernels)

namespace llmem {

void set_error_text(const char *text);          // estimate.hip: what llmem_strerror(LLMEM_EHIP) returns
const char *last_hip_error();

namespace {

// waves per SIMD the build aims at: five (96 registers) for one architecture; with several, the
// code of each sits in a loop over the architectures and needs more registers
inline int specialized_waves(size_t n_arch) { return n_arch == 1 ? 5 : 3; }
// how many times the resident workgroups a launch may have (lane_kernel_blocks): with the detail columns a
// launch is level with its memory traffic, which runs best with a batch per wavefront (measured on 10^7
// configurations: 16 x 0.277, 48 x 0.271 ms; m_peak alone, bound by arithmetic: 0.1125 against 0.115 ms)
inline int specialized_spread(int flavour) { return flavour == 1 ? 48 : 16; }
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

// One per key.  The thread that creates it builds the kernel WITHOUT holding g_lock, so that
// launches of kernels that are already built (other keys) go on meanwhile; threads that want
// the same key wait for `done`.
struct Slot {
    bool done = false;
    int rc = LLMEM_OK;
    std::string problem;
    Built built;
    unsigned long long used = 0;                // g_clock at the last call that looked it up
};

std::mutex g_lock;
std::condition_variable g_built_changed;
unsigned long long g_clock = 0;

// How many kernels built at run time a process keeps loaded per device (LLMEM_KERNELS_KEPT, at
// least 2): a process that goes through table sets without end does not collect modules without end.
int kept_limit()
{
    static const int limit = [] {
        const char *text = getenv("LLMEM_KERNELS_KEPT");
        const int n = text && text[0] ? atoi(text) : 64;
        return n < 2 ? 2 : n;
    }();
    return limit;
}

void unload(Built &built)
{
    if (built.module) (void)hipModuleUnload(built.module);
    built.module = nullptr;
    built.function = nullptr;
    delete built.code;
    built.code = nullptr;
}
std::map<Key, std::shared_ptr<Slot>> g_built;   // finished builds stay (modules loaded) until release_built() or the process ends

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

// specialized_prog.h of a run-time build: the constants estimate_batch.hip declares its tables from
std::string constants_header(const Key &key)
{
    const std::vector<uint32_t> &words = key.words;
    std::string list;
    char item[16];
    for (size_t q = 0; q < words.size(); ++q) {
        snprintf(item, sizeof(item), "0x%08xu,", words[q]);
        list += item;
        if (q % 8 == 7) list += " \\\n";
    }
    std::string firsts;
    for (size_t q = 0; q < 8; ++q) firsts += std::to_string(q < key.first.size() ? key.first[q] : 0) + (q < 7 ? ", " : "");
    return "#pragma once\n#define LLMEM_SPEC_WAVES " + std::to_string(specialized_waves(key.first.size()))
           + "\n#define LLMEM_SPEC_ARCHS " + std::to_string(key.first.size()) + "\n#define LLMEM_SPEC_FIRSTS " + firsts
           + "\n#define LLMEM_SPEC_WORDS \\\n" + list + "\n";
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
    std::string id = std::string("llmem-specialized-3|") + arch_name + "|" + std::to_string(key.flavour) + "|"
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

// The run-time compiler has crashed the process when started under rocprofv3 (its tool library
// preloaded): such a process only loads kept code objects.  Returns the variable that gives the
// profiler away, or null.
const char *profiler_loaded()
{
    const char *tools = getenv("ROCP_TOOL_LIBRARIES");
    if (tools && tools[0]) return "ROCP_TOOL_LIBRARIES";
    const char *preload = getenv("LD_PRELOAD");
    if (preload && strstr(preload, "rocprofiler-sdk-tool")) return "LD_PRELOAD";
    const char *hsa_tools = getenv("HSA_TOOLS_LIB");
    if (hsa_tools && strstr(hsa_tools, "rocprof")) return "HSA_TOOLS_LIB";
    return nullptr;
}

int refuse_under_profiler(const char *tool)
{
    return fail(std::string("the run-time compiler is not started inside a profiled process (") + tool
                + " names a profiler): run once unprofiled with LLMEM_KERNEL_CACHE naming a directory and profile with "
                  "the same directory, or use tables the library has a built-in specialization for");
}

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
            if (const char *tool = profiler_loaded()) {
                delete out->code;
                out->code = nullptr;
                return refuse_under_profiler(tool);
            }
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

// the kernel built into the library for exactly these compiled tables and this flavour, or null
const Prebuilt *find_prebuilt(const EstimateArgs &args, int flavour)
{
    const size_t n_words = words_used(args);
    for (int q = 0; q < PREBUILT_COUNT; ++q) {
        const Prebuilt &p = PREBUILT[q];
        if (p.flavour != flavour || p.n_arch != args.n_arch || (size_t)p.n_words != n_words) continue;
        bool same = true;
        for (int ar = 0; ar < args.n_arch && same; ++ar) same = p.first[ar] == args.arch[ar].prog_first;
        if (same && memcmp(p.words, args.prog, n_words * sizeof(uint32_t)) == 0) return &p;
    }
    return nullptr;
}

}  // namespace

bool has_prebuilt(const EstimateArgs &args, int flavour)
{
    return args.use_program && flavour >= 0 && flavour <= 2 && find_prebuilt(args, flavour) != nullptr;
}

namespace {

constexpr int DEVICES_MAX = 64;

int launch_prebuilt(const Prebuilt &p, const EstimateArgs &args, long long n_batch, hipStream_t stream)
{
    const size_t lds_bytes = batch_kernel_lds_bytes(args);
    const void *kernel = p.entry();
    // resident workgroups per compute unit and compute units, asked once per kernel and device
    static std::atomic<int> resident_of[DEVICES_MAX][sizeof(PREBUILT) / sizeof(PREBUILT[0])];
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return fail("no current device");
    const int slot = device >= 0 && device < DEVICES_MAX ? device : 0;
    int resident = resident_of[slot][&p - PREBUILT].load(std::memory_order_relaxed);
    if (resident == 0) {
        int per_cu = 0, cu_count = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 64 * args.waves, lds_bytes) != hipSuccess || per_cu < 1)
            per_cu = 1;
        if (hipDeviceGetAttribute(&cu_count, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cu_count < 1)
            cu_count = 256;
        resident = per_cu * cu_count;
        resident_of[slot][&p - PREBUILT].store(resident, std::memory_order_relaxed);
    }
    const long long blocks = lane_kernel_blocks(n_batch, args.waves, resident, specialized_spread(p.flavour), p.flavour == 2);
    EstimateArgs copy = args;
    void *params[] = {&copy};
    const hipError_t e = hipLaunchKernel(kernel, dim3((unsigned)blocks), dim3(64 * args.waves), params, lds_bytes, stream);
    if (e != hipSuccess) return fail(std::string("launching the built-in specialized kernel: ") + hipGetErrorString(e));
    return LLMEM_OK;
}

}  // namespace

int launch_specialized(const EstimateArgs &args, int flavour, long long n_batch, hipStream_t stream, bool at_run_time)
{
    if (flavour < 0 || flavour > 2 || !args.use_program || args.n_arch < 1 || args.n_arch > LLMEM_MAX_ARCH)
        return LLMEM_EINVAL_TABLE;
    if (!at_run_time) {
        if (const Prebuilt *p = find_prebuilt(args, flavour)) return launch_prebuilt(*p, args, n_batch, stream);
    }
    // a profiled process may only load kept code objects: without a place to keep them there is
    // nothing to try (decided before any device or compiler call)
    if (const char *tool = profiler_loaded()) {
        const char *dir = getenv("LLMEM_KERNEL_CACHE");
        if (!dir || !dir[0]) return refuse_under_profiler(tool);
    }
    Key key;
    if (hipGetDevice(&key.device) != hipSuccess) return fail("no current device");
    key.flavour = flavour;
    for (int q = 0; q < args.n_arch; ++q) key.first.push_back(args.arch[q].prog_first);
    key.words.assign(args.prog, args.prog + words_used(args));
    const size_t lds_bytes = batch_kernel_lds_bytes(args);
    std::shared_ptr<Slot> slot;
    std::vector<std::shared_ptr<Slot>> evicted;
    bool mine = false;
    {
        std::unique_lock<std::mutex> hold(g_lock);
        auto at = g_built.find(key);
        if (at == g_built.end()) {
            // room for one more on this device?  Else the less recently used half of the finished
            // builds that no call is holding leaves the list now and is unloaded below
            std::vector<std::pair<unsigned long long, const Key *>> idle;
            int kept = 0;
            for (auto &entry : g_built) {
                if (entry.first.device != key.device || !entry.second->done) continue;
                ++kept;
                if (entry.second.use_count() == 1) idle.emplace_back(entry.second->used, &entry.first);
            }
            if (kept >= kept_limit()) {
                std::sort(idle.begin(), idle.end());
                idle.resize(idle.size() < (size_t)(kept + 1) / 2 ? idle.size() : (size_t)(kept + 1) / 2);
                std::vector<Key> keys;
                for (auto &entry : idle) keys.push_back(*entry.second);
                for (const Key &k : keys) {
                    auto victim = g_built.find(k);
                    evicted.push_back(victim->second);
                    g_built.erase(victim);
                }
            }
            slot = std::make_shared<Slot>();
            slot->used = ++g_clock;
            g_built.emplace(key, slot);
            mine = true;
        } else {
            slot = at->second;
            slot->used = ++g_clock;
            g_built_changed.wait(hold, [&] { return slot->done; });
        }
    }
    if (!evicted.empty()) {
        // launches of the kernels that leave may still be pending: they have ended after this
        (void)hipDeviceSynchronize();
        for (auto &gone : evicted) unload(gone->built);
    }
    if (mine) {
        // built outside the lock: seconds, during which other kernels are found and launched
        Built built;
        int rc = build(key, &built);
        std::string problem = rc == LLMEM_OK ? std::string() : std::string(llmem::last_hip_error());
        if (rc == LLMEM_OK) {
            int per_cu = 0;
            if (hipModuleOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, built.function, 64 * args.waves, lds_bytes)
                    == hipSuccess && per_cu > 0)
                built.per_cu = per_cu;
        }
        {
            std::lock_guard<std::mutex> hold(g_lock);
            slot->built = built;
            slot->rc = rc;
            slot->problem = problem;
            slot->done = true;
            if (rc != LLMEM_OK) g_built.erase(key);                  // a later call tries again
        }
        g_built_changed.notify_all();
    }
    if (slot->rc != LLMEM_OK) {
        if (!mine) set_error_text(slot->problem.c_str());             // the error text is per thread
        return slot->rc;
    }
    const Built &built = slot->built;
    const long long blocks = lane_kernel_blocks(n_batch, args.waves, (long long)built.per_cu * built.cu_count, specialized_spread(flavour), flavour == 2);
    EstimateArgs copy = args;
    void *params[] = {&copy};
    const hipError_t e = hipModuleLaunchKernel(built.function, (unsigned)blocks, 1, 1, 64 * args.waves, 1, 1,
                                               (unsigned)lds_bytes, stream, params, nullptr);
    if (e != hipSuccess) return fail(std::string("launching the specialized kernel: ") + hipGetErrorString(e));
    return LLMEM_OK;
}

// Unloads the modules of all finished run-time builds and frees their code objects; builds that
// are still running, and kernels that a call of another thread is about to launch, are left
// alone.  Each device is synchronized before its modules go, so launches that are still
// pending have ended.  Returns how many kernels were released.
int release_built()
{
    std::vector<std::pair<int, std::shared_ptr<Slot>>> gone;
    {
        std::lock_guard<std::mutex> hold(g_lock);
        for (auto at = g_built.begin(); at != g_built.end();) {
            // use_count 1: only the list holds it, and nobody takes it without g_lock
            if (at->second->done && at->second.use_count() == 1) {
                gone.emplace_back(at->first.device, at->second);
                at = g_built.erase(at);
            } else {
                ++at;
            }
        }
    }
    if (gone.empty()) return 0;                                 // nothing built: no device call at all
    int current = 0, count = 0, synchronized = -1;
    const bool restore = hipGetDevice(&current) == hipSuccess;
    for (auto &entry : gone) {                                  // in the order of the keys: device by device
        Built &built = entry.second->built;
        if (entry.second->rc != LLMEM_OK || !built.module) continue;
        if (hipSetDevice(entry.first) != hipSuccess) continue;
        if (synchronized != entry.first) {
            (void)hipDeviceSynchronize();
            synchronized = entry.first;
        }
        unload(built);
        ++count;
    }
    if (restore) (void)hipSetDevice(current);
    return count;
}

}  // namespace llmem
