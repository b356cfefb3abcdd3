// Library-internal state: blob layout, chunk plan, residency, staging slots, events, the
// prefetch worker and the per-kernel profiler.  Not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <condition_variable>
#include <deque>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "../../include/chunkflow.h"
#include "../../include/chunkflow_diag.h"
#include "kernels.h"

struct TensorDesc {
    std::string name;
    uint64_t off;
    uint32_t rows, cols;
    uint64_t bytes() const { return 2ull * rows * cols; }
};

struct ProfEntry {
    int kid;
    hipEvent_t a, b;
    double flops, bytes;
};

enum { SLOT_EMPTY = 0, SLOT_FILLED = 1, SLOT_CONSUMED = 2 };

// A collective announced by cf_comm_begin that the prefetch worker has not yet seen finished (Sec. 3.2):
// `ready` fires when the compute stream reaches the collective, `done` when the collective has finished.
struct PendingComm {
    hipEvent_t ready, done;
    bool done_recorded;     // cf_comm_end has recorded `done` on the collective's stream
    bool handled;           // the copy stream has already been parked on `done`
};

struct PrefetchJob {
    int block;
    int slot;
    hipStream_t copy;
};

// Blob layout, chunk plan and residency of one block kind (a model may mix kinds, App. B:
// double-stream blocks followed by single-stream ones)
struct Plan {
    int kind = -1;
    std::vector<TensorDesc> tensors;
    uint64_t blob_bytes = 0;
    int n_chunks = 0;
    // residency (Sec. 3.3): the leading n_res_chunks chunks of every block of this kind stay in HBM
    int n_res_chunks = 0;
    uint64_t res_bytes = 0;
    uint64_t ws_bytes = 0;
};

struct cf_ctx {
    cf_model_desc d{};
    uint64_t chunk_bytes = 0;
    Plan plan[3];                       // indexed by cf_block_kind; kind < 0 = not used by this model
    std::vector<int> block_kind;
    uint64_t ws_bytes = 0;              // largest over the kinds in use
    int max_chunks = 0;
    const Plan& P(int block) const { return plan[block_kind[block]]; }

    std::vector<const uint8_t*> host;
    std::vector<uint8_t*> res_buf;

    // staging (Sec. 2.2: two layers live) -- slot s holds blob bytes [res_bytes, blob) of its tenant;
    // slots are sized for the kind with the most streamed bytes
    bool device_ready = false;
    int device = 0;
    uint8_t* slot[2] = {nullptr, nullptr};
    int slot_tenant[2] = {-1, -1};
    std::vector<int> block_slot;        // slot holding the block's streamed bytes, or -1
    int next_slot = 0;                  // slots alternate per prefetch
    int slot_state[2] = {SLOT_EMPTY, SLOT_EMPTY};
    std::vector<hipEvent_t> chunk_ev[2];
    hipEvent_t done_ev[2] = {nullptr, nullptr};
    std::atomic<bool> done_valid[2] = {{false}, {false}};     // read by the prefetch worker
    int waited_upto = -1;               // highest chunk the current forward already waited for
    // One wait per block when the prefetch is hidden anyway: land_ev[s] follows the last chunk copy into
    // slot s; comparing it with the end of the block that ran before the slot's tenant tells whether that
    // tenant's weights had landed before it started (Sec. 3.1: T_pref <= T_comp), per block kind.
    hipEvent_t land_ev[2] = {nullptr, nullptr};
    std::atomic<bool> land_valid[2] = {{false}, {false}};     // written by the prefetch worker
    uint64_t fwd_seq = 0, slot_fwd_seq[2] = {0, 0};   // order of the forwards that recorded done_ev[s]
    bool adaptive_waits = true;
    bool hidden_kind[3] = {false, false, false};

    // emulated collectives + pause/resume (Sec. 3.2)
    hipStream_t comm_stream = nullptr;
    uint8_t* comm_host = nullptr;
    uint8_t* comm_dev = nullptr;
    uint64_t comm_bytes = 0;
    bool pause_resume = false;
    int pause_depth = 1;                // chunk copies the worker keeps enqueued ahead of the link in pause/resume mode
    hipEvent_t comm_ready_ev = nullptr, comm_done_ev = nullptr;   // the one pair used without pause/resume
    hipEvent_t cur_ready = nullptr, cur_done = nullptr;           // the pair of the collective being issued
    std::deque<PendingComm> comm_pending;      // guarded by mu; oldest first
    std::vector<hipEvent_t> comm_ev_pool;      // guarded by mu; events of retired collectives
    // Host run-ahead bound while collectives are emulated: forward n is enqueued once forward n-2 has finished.
    hipEvent_t fwd_ev[4] = {nullptr, nullptr, nullptr, nullptr};
    uint64_t fwd_count = 0;

    std::thread worker;
    std::mutex mu;
    std::condition_variable cv;
    std::deque<PrefetchJob> jobs;
    bool worker_stop = false, worker_busy = false;
    int enq_count[2] = {0, 0};          // chunks of the slot's tenant whose copy has been enqueued
    std::string worker_err;

    uint64_t* checksum_dev = nullptr;   // max_chunks words for cf_checksum_block, allocated at its first call

    // statistics / profiling
    cf_stats_t stats{};
    bool profiling = false;
    std::vector<ProfEntry> prof_pending;
    std::vector<hipEvent_t> ev_pool;
    std::vector<cf_kernel_time> ktimes;

    mutable std::string err;
};

const TensorDesc* cf_find(const Plan& p, const char* name);
// records the message in the context (or, with none, for cf_last_error(NULL)) and returns `code`
int cf_fail(const cf_ctx* c, int code, const char* fmt, ...);
// blob layout and chunk count of one block kind
void plan_layout(Plan* p, const cf_model_desc& m, int kind, uint64_t chunk_bytes);

#define CF_TRY(expr)                  \
    do {                              \
        int rc_ = (expr);             \
        if (rc_ != CF_OK) return rc_; \
    } while (0)
