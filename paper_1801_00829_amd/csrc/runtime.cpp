#include "runtime.h"

#include <hip/hiprtc.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "../../include/fuse.h"

namespace fuse {

Runtime &Runtime::get()
{
    static Runtime *r = new Runtime();   // never destroyed: HIP may be gone at exit
    return *r;
}

std::string Runtime::hash_hex(const std::string &s)
{
    uint64_t h = 1469598103934665603ull;   // FNV-1a
    for (unsigned char c : s) {
        h ^= c;
        h *= 1099511628211ull;
    }
    char buf[20];
    std::snprintf(buf, sizeof buf, "%016llx", (unsigned long long)h);
    return buf;
}

std::string Runtime::arch()
{
    std::lock_guard<std::mutex> lk(mu_);
    if (!arch_.empty())
        return arch_;
    if (const char *e = std::getenv("FUSE_ARCH")) {
        arch_ = e;
        return arch_;
    }
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
            prop.gcnArchName[0])
            arch_ = prop.gcnArchName;
    } else {
        (void)hipGetLastError();
    }
    if (arch_.empty())
        arch_ = "gfx950";
    return arch_;
}

namespace {

// On-disk copies of compiled code objects (FUSE_CACHE_DIR): "FUSECO01", payload length, FNV-1a of the
// payload, payload.  A file that does not check out is ignored and rewritten.
const char kDiskMagic[8] = {'F', 'U', 'S', 'E', 'C', 'O', '0', '1'};

uint64_t fnv1a(const char *d, size_t n)
{
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < n; ++i) {
        h ^= (unsigned char)d[i];
        h *= 1099511628211ull;
    }
    return h;
}

bool disk_read(const std::string &path, std::vector<char> &code)
{
    std::FILE *f = std::fopen(path.c_str(), "rb");
    if (!f)
        return false;
    char magic[8];
    uint64_t len = 0, sum = 0;
    bool ok = std::fread(magic, 1, 8, f) == 8 && std::memcmp(magic, kDiskMagic, 8) == 0 &&
              std::fread(&len, sizeof len, 1, f) == 1 && std::fread(&sum, sizeof sum, 1, f) == 1 && len > 0 &&
              len < (1ull << 30);
    if (ok) {
        code.resize((size_t)len);
        ok = std::fread(code.data(), 1, (size_t)len, f) == (size_t)len && std::fgetc(f) == EOF &&
             fnv1a(code.data(), (size_t)len) == sum;
    }
    std::fclose(f);
    if (!ok)
        code.clear();
    return ok;
}

void disk_write(const std::string &path, const std::vector<char> &code)
{
    // written under a name of its own and renamed: readers see a whole file or none
    const std::string tmp = path + ".tmp" + std::to_string((unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count());
    std::FILE *f = std::fopen(tmp.c_str(), "wb");
    if (!f)
        return;
    const uint64_t len = code.size(), sum = fnv1a(code.data(), code.size());
    const bool ok = std::fwrite(kDiskMagic, 1, 8, f) == 8 && std::fwrite(&len, sizeof len, 1, f) == 1 &&
                    std::fwrite(&sum, sizeof sum, 1, f) == 1 && std::fwrite(code.data(), 1, code.size(), f) == code.size();
    if (std::fclose(f) != 0 || !ok || std::rename(tmp.c_str(), path.c_str()) != 0)
        std::remove(tmp.c_str());
}

}  // namespace

int Runtime::compile(Plan &p, std::string &err)
{
    const auto t0 = std::chrono::steady_clock::now();
    const std::string arch_opt = "--offload-arch=" + arch();
    // -ffp-contract=off: a body rounds after every operator, exactly like the chain of
    // basic operators it replaces (a*b+c is not silently turned into one fused
    // multiply-add); the skeletons call fma() explicitly where they want one.
    const char *opts[] = {arch_opt.c_str(), "-O3", "-std=c++17", "-Xclang", "-target-feature",
                          "-Xclang", "-packed-fp32-ops", "-munsafe-fp-atomics", "-ffp-contract=off"};
    // FUSE_CACHE_DIR: code objects are kept there across processes, named by the kernel and a hash of
    // the source text, the options and the compiler's version
    std::string disk_path;
    if (const char *dir = std::getenv("FUSE_CACHE_DIR")) {
        if (*dir) {
            int major = 0, minor = 0;
            (void)hiprtcVersion(&major, &minor);
            std::string id = p.source + "\n";
            for (const char *o : opts)
                id += std::string(o) + " ";
            id += "hiprtc " + std::to_string(major) + "." + std::to_string(minor);
            disk_path = std::string(dir) + "/" + p.kernel_name + "-" + hash_hex(id) + ".co";
            if (disk_read(disk_path, p.code)) {
                std::lock_guard<std::mutex> lk(mu_);
                ++disk_hits_;
                return 0;
            }
        }
    }
    hiprtcProgram prog;
    hiprtcResult r = hiprtcCreateProgram(&prog, p.source.c_str(), (p.kernel_name + ".hip").c_str(), 0,
                                         nullptr, nullptr);
    if (r != HIPRTC_SUCCESS) {
        err = std::string("hiprtcCreateProgram: ") + hiprtcGetErrorString(r);
        return FUSE_ECOMPILE;
    }
    r = hiprtcCompileProgram(prog, (int)(sizeof opts / sizeof opts[0]), opts);
    if (r != HIPRTC_SUCCESS) {
        size_t n = 0;
        hiprtcGetProgramLogSize(prog, &n);
        std::string log(n, '\0');
        if (n)
            hiprtcGetProgramLog(prog, &log[0]);
        err = std::string("hipRTC: ") + hiprtcGetErrorString(r) + "\n" + log;
        hiprtcDestroyProgram(&prog);
        return FUSE_ECOMPILE;
    }
    size_t n = 0;
    hiprtcGetCodeSize(prog, &n);
    p.code.resize(n);
    hiprtcGetCode(prog, p.code.data());
    hiprtcDestroyProgram(&prog);
    if (!disk_path.empty())
        disk_write(disk_path, p.code);
    const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    std::lock_guard<std::mutex> lk(mu_);
    compile_ms_ += ms;
    return 0;
}

int Runtime::load(Plan &p, Plan::Loaded &fn, std::string &err)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        err = std::string("hipGetDevice: ") + hipGetErrorString(e);
        return FUSE_ERUNTIME;
    }
    std::lock_guard<std::mutex> lk(p.mu);
    auto it = p.per_device.find(dev);
    if (it != p.per_device.end()) {
        fn = it->second;
        return 0;
    }
    Plan::Loaded l;
    e = hipModuleLoadData(&l.module, p.code.data());
    if (e != hipSuccess) {
        err = std::string("hipModuleLoadData: ") + hipGetErrorString(e);
        return FUSE_ERUNTIME;
    }
    e = hipModuleGetFunction(&l.main, l.module, p.kernel_name.c_str());
    if (e == hipSuccess)
        e = hipModuleGetFunction(&l.combine, l.module, "fuse_combine_cols");
    if (e == hipSuccess)
        e = hipModuleGetFunction(&l.fill, l.module, "fuse_fill");
    if (e == hipSuccess && p.source.find("void __launch_bounds__(256) fuse_outer_prep") != std::string::npos &&
        (p.source.find("#define FUSE_PANELS 1") != std::string::npos || p.source.find("#define FUSE_PANELS 2") != std::string::npos ||
         p.source.find("#define FUSE_PANELS 3") != std::string::npos))
        e = hipModuleGetFunction(&l.prep, l.module, "fuse_outer_prep");
    if (e != hipSuccess) {
        err = std::string("hipModuleGetFunction: ") + hipGetErrorString(e);
        (void)hipModuleUnload(l.module);
        return FUSE_ERUNTIME;
    }
    p.per_device[dev] = l;
    fn = l;
    return 0;
}

bool Runtime::find_plan(const std::string &key, std::shared_ptr<Plan> &out)
{
    std::lock_guard<std::mutex> lk(mu_);
    auto it = plans_.find(key);
    if (it == plans_.end())
        return false;
    ++hits_;
    out = it->second;
    return true;
}

bool Runtime::loaded(Plan &p, Plan::Loaded &fn)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return false;
    std::lock_guard<std::mutex> lk(p.mu);
    auto it = p.per_device.find(dev);
    if (it == p.per_device.end())
        return false;
    fn = it->second;
    return true;
}

int Runtime::workspace(hipStream_t stream, size_t doubles, Workspace &ws, std::string &err)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        err = std::string("hipGetDevice: ") + hipGetErrorString(e);
        return FUSE_ERUNTIME;
    }
    std::lock_guard<std::mutex> lk(mu_);
    Workspace &w = ws_[std::make_pair(dev, stream)];
    if (!w.ticket) {
        e = hipMalloc((void **)&w.ticket, 256);
        if (e == hipSuccess && reset_ticket_launch(w.ticket, stream))     // cleared on the caller's stream, no host sync
            e = hipErrorLaunchFailure;
        if (e != hipSuccess) {
            if (w.ticket)
                (void)hipFree(w.ticket);
            w.ticket = nullptr;
            err = std::string("workspace ticket: ") + hipGetErrorString(e);
            return FUSE_ENOMEM;
        }
    }
    // (also for a request of 0 doubles on a stream without a workspace yet: callers use the buffer's
    //  address, e.g. as the one dummy cell of a CSR matrix without stored cells, and it must never be null)
    if (!w.partials || w.partial_doubles < doubles) {
        size_t want = doubles < 65536 ? 65536 : doubles + doubles / 4;
        double *np = nullptr;
        e = hipMalloc((void **)&np, want * sizeof(double));
        if (e != hipSuccess) {
            err = std::string("workspace partials: ") + hipGetErrorString(e);
            return FUSE_ENOMEM;
        }
        if (w.partials)
            retired_.push_back(w.partials);   // may still be read by work in flight
        w.partials = np;
        w.partial_doubles = want;
    }
    ws = w;
    return 0;
}

int Runtime::resident_blocks_per_cu(hipFunction_t f, int block)
{
    std::lock_guard<std::mutex> lk(mu_);
    auto key = std::make_pair(f, block);
    auto it = resident_.find(key);
    if (it != resident_.end())
        return it->second;
    int nb = 0;
    if (hipModuleOccupancyMaxActiveBlocksPerMultiprocessor(&nb, f, block, 0) != hipSuccess || nb < 1) {
        (void)hipGetLastError();
        nb = 1;
    }
    resident_[key] = nb;
    return nb;
}

int Runtime::launch(hipFunction_t f, unsigned gx, unsigned gy, unsigned block, hipStream_t stream,
                    const void *args, size_t arg_bytes, std::string &err)
{
    if (gx == 0 || gy == 0 || block == 0)       // nothing to do; an empty grid is not a valid launch
        return 0;
    if (gx > 2147483647u || gy > 65535u || block > 1024u) {
        err = "internal: launch shape out of range (" + std::to_string(gx) + " x " + std::to_string(gy) + " blocks of " +
              std::to_string(block) + " threads)";
        return FUSE_ERUNTIME;
    }
    void *config[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, const_cast<void *>(args),
                      HIP_LAUNCH_PARAM_BUFFER_SIZE, &arg_bytes, HIP_LAUNCH_PARAM_END};
    hipError_t e = hipModuleLaunchKernel(f, gx, gy, 1, block, 1, 1, 0, stream, nullptr, config);
    if (e != hipSuccess) {
        err = std::string("hipModuleLaunchKernel: ") + hipGetErrorString(e);
        return FUSE_ERUNTIME;
    }
    return 0;
}

int Runtime::num_cus()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return 256;
    std::lock_guard<std::mutex> lk(mu_);
    auto it = cus_.find(dev);
    if (it != cus_.end())
        return it->second;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        n = 256;
    cus_[dev] = n;
    return n;
}

void Runtime::stats(int64_t *hits, int64_t *misses, double *ms)
{
    std::lock_guard<std::mutex> lk(mu_);
    if (hits)
        *hits = hits_;
    if (misses)
        *misses = misses_;
    if (ms)
        *ms = compile_ms_;
}

int64_t Runtime::disk_hits()
{
    std::lock_guard<std::mutex> lk(mu_);
    return disk_hits_;
}

void Runtime::clear()
{
    std::lock_guard<std::mutex> lk(mu_);
    for (auto &kv : plans_)
        for (auto &d : kv.second->per_device)
            if (d.second.module)
                (void)hipModuleUnload(d.second.module);
    plans_.clear();
    resident_.clear();
    for (auto &kv : ws_) {
        if (kv.second.partials)
            (void)hipFree(kv.second.partials);
        if (kv.second.ticket)
            (void)hipFree(kv.second.ticket);
    }
    ws_.clear();
    for (void *p : retired_)
        (void)hipFree(p);
    retired_.clear();
    hits_ = misses_ = disk_hits_ = 0;
    compile_ms_ = 0.0;
}

}  // namespace fuse
