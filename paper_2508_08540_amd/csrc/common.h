// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string>
#include <vector>

#include "../../include/bls.h"

// Kernel classes for the optional per-class timing (bls_profile_begin / bls_profile_end).
enum ProfClass { PROF_CONV_FWD = 0, PROF_CONV_DGRAD, PROF_CONV_WGRAD, PROF_NORM, PROF_HEAD, PROF_GEMM, PROF_UPDATE,
                 PROF_GATHER, PROF_TOPK, PROF_AGGREGATE, PROF_WGRAD_REDUCE, PROF_NUM_CLASSES };

struct ProfSpan {
    int cls;
    hipEvent_t start, stop;
};

struct bls_ctx {
    bool profiling = false;
    std::vector<ProfSpan> spans;
    int device = 0;
    hipStream_t stream = nullptr;
    hipStream_t aux = nullptr;             // library-owned side stream for work off the critical path
    hipStream_t aux2 = nullptr;            // a second one, created on first use: bf16 ResNet weight gradients alternate between the two
    std::vector<hipEvent_t> fork_events;   // main -> aux dependencies, one per use inside a call
    hipEvent_t join_event = nullptr;       // aux -> main
    hipEvent_t join_event2 = nullptr;      // aux2 -> main
    hipEvent_t head_event = nullptr;       // main -> aux: the classifier head's gradients are written
    float* round_losses = nullptr;   // per-sample losses of the workers' local steps (communication_round), grown on demand
    size_t round_losses_count = 0;
    std::vector<bls_ctx*> lanes;     // library-owned contexts (own stream, side stream and scratch) for concurrent workers
    std::vector<hipEvent_t> lane_events;   // one per worker of a round: its local steps are done
    hipEvent_t round_start = nullptr;      // main stream -> lanes
    bool owns_stream = false;
    char* arena = nullptr;      // one scratch allocation, grown on demand
    size_t arena_bytes = 0;
    int num_cus = 0;
    size_t max_lds = 0;
    std::string error;
};

int bls_fail(bls_ctx* ctx, int code, const char* fmt, ...);

#define BLS_HIP(ctx, expr)                                                                  \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            return bls_fail((ctx), BLS_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// Brackets the launches issued during its lifetime with HIP events when profiling is on.
struct ProfScope {
    bls_ctx* ctx;
    ProfSpan span;
    bool on;
    hipStream_t st;
    ProfScope(bls_ctx* c, int cls, hipStream_t stream = nullptr) : ctx(c), on(c->profiling), st(stream ? stream : c->stream) {
        if (!on) return;
        span.cls = cls;
        if (hipEventCreate(&span.start) != hipSuccess || hipEventCreate(&span.stop) != hipSuccess) {
            on = false;
            return;
        }
        (void)hipEventRecord(span.start, st);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(span.stop, st);
        ctx->spans.push_back(span);
    }
};

// Timing of exactly one kernel: the events are attached to the dispatch by the launcher.
struct ProfKernel {
    bls_ctx* ctx;
    ProfSpan span;
    bool on;
    ProfKernel(bls_ctx* c, int cls) : ctx(c), on(c->profiling) {
        if (!on) return;
        span.cls = cls;
        if (hipEventCreate(&span.start) != hipSuccess || hipEventCreate(&span.stop) != hipSuccess) on = false;
    }
    ~ProfKernel() {
        if (on) ctx->spans.push_back(span);
    }
};

// Makes the context's scratch arena at least `bytes` large.  Growing waits for the stream first.
int bls_arena_reserve(bls_ctx* ctx, size_t bytes);

// Bump allocator over the arena; every block is 256-byte aligned.
struct Carver {
    char* base;
    size_t off = 0;
    explicit Carver(char* b) : base(b) {}
    template <typename T>
    T* take(size_t count) {
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += (count * sizeof(T) + 255) & ~size_t(255);
        return p;
    }
};

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- launchers (each enqueues on ctx->stream and returns a bls_status) ------------------------
int launch_weighted_aggregate(bls_ctx* ctx, const float* const* replicas, const float* weights, int P, int64_t d,
                              float* out, bool broadcast);
size_t topk_scratch_bytes(int64_t N, int64_t k);
int launch_topk(bls_ctx* ctx, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out);
// The same on the library's fixed device array (no allocation); topk_static_init looks its address up for ctx's device.
int topk_static_init(bls_ctx* ctx);
int launch_topk_static(bls_ctx* ctx, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out);
int launch_sample_epoch(bls_ctx* ctx, const float* losses, const float* u_biased, const float* u_other, int64_t N, int64_t n_biased,
                        int64_t k, int64_t n_other, int P_biased, int P_other, bool unified, int32_t* biased_out, int32_t* other_out);
