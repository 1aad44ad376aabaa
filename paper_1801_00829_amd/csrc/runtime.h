// hipRTC compilation, plan cache, per-stream workspaces and kernel launch.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <map>
#include <memory>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "fuse_args.h"

namespace fuse {

// One compiled body + skeleton (a "generated operator class" of Sec. 2.1).
struct Plan {
    std::string kernel_name;
    std::string source;
    std::vector<char> code;                 // gfx950 code object from hipRTC
    std::mutex mu;
    struct Loaded {
        hipModule_t module = nullptr;
        hipFunction_t main = nullptr;
        hipFunction_t combine = nullptr;    // fuse_combine_cols
        hipFunction_t fill = nullptr;       // fuse_fill
        hipFunction_t prep = nullptr;       // fuse_outer_prep (Outer plans with column panels only)
    };
    std::map<int, Loaded> per_device;
};

struct Workspace {
    double *partials = nullptr;
    size_t partial_doubles = 0;
    unsigned int *ticket = nullptr;
};

class Runtime {
public:
    static Runtime &get();

    // Look up `key`; on a miss build the source with `make_source(kernel_name)`
    // and compile it.  Returns FUSE_OK / FUSE_ECOMPILE (message in err).
    template <typename F>
    int plan(const std::string &key, const std::string &name_prefix, F make_source,
             std::shared_ptr<Plan> &out, std::string &err)
    {
        {
            std::lock_guard<std::mutex> lk(mu_);
            auto it = plans_.find(key);
            if (it != plans_.end()) {
                ++hits_;
                out = it->second;
                return 0;
            }
        }
        // The kernel's name carries a hash of the key AND of the source text (generated once under a stand-in
        // name): a profile taken of a kernel names exactly the code it measured.
        const std::string name = name_prefix + "_" + hash_hex(key + "\n" + make_source(name_prefix + "_unnamed"));
        auto p = std::make_shared<Plan>();
        p->kernel_name = name;
        p->source = make_source(name);
        int rc = compile(*p, err);
        if (rc != 0)
            return rc;
        std::lock_guard<std::mutex> lk(mu_);
        ++misses_;
        auto ins = plans_.emplace(key, p);
        out = ins.first->second;
        return 0;
    }

    // Look up `key` only: false when no plan with that key has been compiled (nothing is compiled here).
    bool find_plan(const std::string &key, std::shared_ptr<Plan> &out);
    // Load (once per device) and return the functions of a plan on the current device.
    int load(Plan &p, Plan::Loaded &fn, std::string &err);
    // The functions of a plan if it is already loaded on the current device (nothing is loaded here).
    bool loaded(Plan &p, Plan::Loaded &fn);
    // Workspace of (current device, stream) with room for `doubles` partials.
    int workspace(hipStream_t stream, size_t doubles, Workspace &ws, std::string &err);
    // Workgroups of `block` threads of kernel `f` that one compute unit holds at once (>= 1).
    int resident_blocks_per_cu(hipFunction_t f, int block);
    int launch(hipFunction_t f, unsigned gx, unsigned gy, unsigned block, hipStream_t stream,
               const void *args, size_t arg_bytes, std::string &err);

    int num_cus();
    void stats(int64_t *hits, int64_t *misses, double *ms);
    int64_t disk_hits();      // code objects taken from FUSE_CACHE_DIR instead of being compiled
    void clear();

    static std::string hash_hex(const std::string &s);

private:
    int compile(Plan &p, std::string &err);
    std::string arch();

    std::mutex mu_;
    std::unordered_map<std::string, std::shared_ptr<Plan>> plans_;
    std::map<std::pair<int, hipStream_t>, Workspace> ws_;
    std::vector<void *> retired_;
    std::map<int, int> cus_;
    std::map<std::pair<hipFunction_t, int>, int> resident_;
    std::string arch_;
    int64_t hits_ = 0, misses_ = 0, disk_hits_ = 0;
    double compile_ms_ = 0.0;
};

// The fixed workspace of the entry point that allocates nothing (noalloc.hip): the current device's copy of
// a file-scope device array, FUSE_NOALLOC_MAX_PARTIALS doubles of block partials behind a zeroed arrival
// counter.  Enqueues one small kernel on `stream` that clears the counter.  0 on success.
int noalloc_workspace(hipStream_t stream, Workspace &ws, std::string &err);
int reset_ticket_launch(unsigned int *ticket, hipStream_t stream);      // 64 words at `ticket` = 0, by a kernel on `stream`

// Launches the CSR structure check (check.hip); `bad` points to four device words, the first
// three preset to all ones and the last to zero.  0 on success.
int check_csr_launch(const void *rowptr, int rowptr_is64, const int *colidx, long long rows, long long cols,
                     long long nnz, unsigned long long *bad, hipStream_t stream);

// Transposition of a CSR matrix (transpose.hip): tptr (n + 1 offsets, of the width of the matrix' own row
// offsets), trow (row of every cell, by column) and tval (its value); `scratch` holds
// transpose_scratch_bytes() bytes, 16-byte aligned.  0 on success.
size_t transpose_scratch_bytes(long long m, long long n, long long nnz, int rowptr_is64);
int transpose_launch(const void *rowptr, int rowptr_is64, const int *colidx, const double *vals, long long m, long long n,
                     long long nnz, void *scratch, void *tptr, int *trow, double *tval, hipStream_t stream);

int iota_launch(double *dst, long long n, hipStream_t stream);     // dst[i] = (double)i
int gather_launch(double *dst, const double *src, const double *perm, long long n, hipStream_t stream);   // dst[i] = src[perm[i]]

}  // namespace fuse
