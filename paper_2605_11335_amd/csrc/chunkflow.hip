// C ABI implementation: layout/chunk planning, residency, chunked prefetch with per-chunk
// events, the pause/resume worker, emulated collectives, and the block forward that strings the
// kernels together.  See include/chunkflow.h for the contract of every entry point.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "context.h"

static std::string g_create_err;
// The prefetch worker reports into a string of its own: the context's message belongs to the
// caller's thread, which may be failing a call of its own at the same moment.
static thread_local std::string* t_err_sink = nullptr;

int cf_fail(const cf_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (t_err_sink) *t_err_sink = buf;
    else if (c) c->err = buf;
    else g_create_err = buf;
    return code;
}

namespace {

#define CF_HIP(c, call)                                                                                  \
    do {                                                                                                 \
        hipError_t e_ = (call);                                                                          \
        if (e_ != hipSuccess) return cf_fail((c), CF_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)
inline uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------------------------------
// blob layout: tensors in the order the block consumes them (small vectors ahead of the matrix
// that needs them), each 256-byte aligned, so a prefix of chunks is a prefix of the computation
// ------------------------------------------------------------------------------------------
void add_tensor(Plan* c, const std::string& name, uint32_t rows, uint32_t cols) {
    TensorDesc t{name, align_up(c->blob_bytes, 256), rows, cols};
    c->blob_bytes = t.off + t.bytes();
    c->tensors.push_back(t);
}

}  // namespace

void plan_layout(Plan* c, const cf_model_desc& m, int kind, uint64_t chunk_bytes) {
    const uint32_t d = m.d, f = m.f, hd = m.head_dim;
    *c = Plan{};
    c->kind = kind;
    if (kind == CF_SINGLE_STREAM) {
        add_tensor(c, "b_mod", 1, 3 * d);
        add_tensor(c, "w_mod", 3 * d, d);
        add_tensor(c, "b1", 1, 3 * d + f);
        if (m.qk_rmsnorm) { add_tensor(c, "q_norm", 1, hd); add_tensor(c, "k_norm", 1, hd); }
        add_tensor(c, "w1", 3 * d + f, d);
        add_tensor(c, "b2", 1, d);
        add_tensor(c, "w2", d, d + f);
    } else if (kind == CF_DIT_CROSS) {
        add_tensor(c, "b_mod", 1, 6 * d);
        add_tensor(c, "w_mod", 6 * d, d);
        add_tensor(c, "b_qkv", 1, 3 * d);
        if (m.qk_rmsnorm) { add_tensor(c, "q_norm", 1, hd); add_tensor(c, "k_norm", 1, hd); }
        add_tensor(c, "w_qkv", 3 * d, d);
        add_tensor(c, "b_o", 1, d);
        add_tensor(c, "w_o", d, d);
        add_tensor(c, "ln_c_w", 1, d);
        add_tensor(c, "ln_c_b", 1, d);
        add_tensor(c, "b_cq", 1, d);
        if (m.qk_rmsnorm) { add_tensor(c, "cq_norm", 1, hd); add_tensor(c, "ck_norm", 1, hd); }
        add_tensor(c, "w_cq", d, d);
        add_tensor(c, "b_ckv", 1, 2 * d);
        add_tensor(c, "w_ckv", 2 * d, d);
        add_tensor(c, "b_co", 1, d);
        add_tensor(c, "w_co", d, d);
        add_tensor(c, "b_up", 1, f);
        add_tensor(c, "w_up", f, d);
        add_tensor(c, "b_down", 1, d);
        add_tensor(c, "w_down", d, f);
    } else {
        static const char* st[2] = {"txt", "img"};
        auto nm = [](const char* s, const char* t) { return std::string(s) + "_" + t; };
        for (int s = 0; s < 2; ++s) { add_tensor(c, nm(st[s], "b_mod"), 1, 6 * d); add_tensor(c, nm(st[s], "w_mod"), 6 * d, d); }
        for (int s = 0; s < 2; ++s) {
            add_tensor(c, nm(st[s], "b_qkv"), 1, 3 * d);
            if (m.qk_rmsnorm) { add_tensor(c, nm(st[s], "q_norm"), 1, hd); add_tensor(c, nm(st[s], "k_norm"), 1, hd); }
            add_tensor(c, nm(st[s], "w_qkv"), 3 * d, d);
        }
        for (int s = 0; s < 2; ++s) { add_tensor(c, nm(st[s], "b_o"), 1, d); add_tensor(c, nm(st[s], "w_o"), d, d); }
        for (int s = 0; s < 2; ++s) {
            add_tensor(c, nm(st[s], "b_up"), 1, f);
            add_tensor(c, nm(st[s], "w_up"), f, d);
            add_tensor(c, nm(st[s], "b_down"), 1, d);
            add_tensor(c, nm(st[s], "w_down"), d, f);
        }
    }
    c->blob_bytes = align_up(c->blob_bytes, 256);
    c->n_chunks = (int)((c->blob_bytes + chunk_bytes - 1) / chunk_bytes);
}

namespace {

// ------------------------------------------------------------------------------------------
// workspace carving (same function plans the size and hands out the pointers)
// ------------------------------------------------------------------------------------------
struct Ws {
    float* mod = nullptr;      // modulation vectors (3d | 6d | 2 x 6d)
    bf16* xn = nullptr;        // [n_local, d]
    bf16* qkv = nullptr;       // [n_local, 3d]
    bf16* c = nullptr;         // single: [n_local, d+f]; others: attention rows [n_local, d]
    bf16 *Q = nullptr, *K = nullptr, *Vt = nullptr;
    float *x1 = nullptr, *x2 = nullptr;
    bf16* up = nullptr;        // [n_local, f]
    bf16 *ckv = nullptr, *cQ = nullptr, *cK = nullptr, *cVt = nullptr;
    uint64_t total = 0;
};

inline int n_pad_of(int n) { return (n + 63) / 64 * 64; }

inline int batch_of(const cf_model_desc& m) { return m.batch > 0 ? m.batch : 1; }

// every per-token buffer holds the whole batch, sample after sample
Ws carve(const cf_model_desc& m, int kind, char* base) {
    Ws w;
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) { char* p = base + off; off = align_up(off + bytes, 256); return p; };
    const uint64_t B = batch_of(m);
    const uint64_t nl = B * (m.n_total / m.sp_degree), d = m.d, f = m.f, N = m.n_total, hd = m.head_dim;
    const uint64_t hl = B * (m.n_heads / m.sp_degree), lc = B * (uint64_t)m.l_ctx;
    const int nmod = kind == CF_SINGLE_STREAM ? 3 : (kind == CF_DIT_CROSS ? 6 : 12);
    w.mod = (float*)take(4ull * B * nmod * d);
    w.xn = (bf16*)take(2 * nl * d);
    w.qkv = (bf16*)take(2 * nl * 3 * d);
    w.c = (bf16*)take(2 * nl * (kind == CF_SINGLE_STREAM ? d + f : d));
    w.Q = (bf16*)take(2 * hl * N * hd);
    w.K = (bf16*)take(2 * hl * N * hd);
    w.Vt = (bf16*)take(2 * hl * hd * n_pad_of(N));
    if (kind != CF_SINGLE_STREAM) {
        w.x1 = (float*)take(4 * nl * d);
        w.up = (bf16*)take(2 * nl * f);
    }
    if (kind == CF_DIT_CROSS) {
        w.x2 = (float*)take(4 * nl * d);
        w.ckv = (bf16*)take(2ull * lc * 2 * d);
        w.cQ = (bf16*)take(2 * nl * d);
        w.cK = (bf16*)take(2ull * lc * d);
        w.cVt = (bf16*)take(2ull * B * d * n_pad_of(m.l_ctx));
    }
    w.total = off;
    return w;
}

// ------------------------------------------------------------------------------------------
// device resources
// ------------------------------------------------------------------------------------------
int ensure_device(cf_ctx* c) {
    if (c->device_ready) return CF_OK;
    CF_HIP(c, hipGetDevice(&c->device));
    for (int s = 0; s < 2; ++s) {
        c->chunk_ev[s].resize(c->max_chunks);
        for (auto& e : c->chunk_ev[s]) CF_HIP(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
        CF_HIP(c, hipEventCreate(&c->done_ev[s]));          // with timestamps: compared with land_ev
        CF_HIP(c, hipEventCreate(&c->land_ev[s]));
    }
    CF_HIP(c, hipEventCreateWithFlags(&c->comm_ready_ev, hipEventDisableTiming));
    CF_HIP(c, hipEventCreateWithFlags(&c->comm_done_ev, hipEventDisableTiming));
    for (auto& e : c->fwd_ev) CF_HIP(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    c->device_ready = true;
    return CF_OK;
}

void free_weights(cf_ctx* c) {
    for (auto& p : c->res_buf) { if (p) (void)hipFree(p); p = nullptr; }
    for (int s = 0; s < 2; ++s) {
        if (c->slot[s]) (void)hipFree(c->slot[s]);
        c->slot[s] = nullptr;
        c->slot_tenant[s] = -1;
        c->slot_state[s] = SLOT_EMPTY;
        c->done_valid[s] = false;
        c->land_valid[s] = false;
        c->enq_count[s] = 0;
    }
    c->next_slot = 0;
    std::fill(c->block_slot.begin(), c->block_slot.end(), -1);
}

int upload_resident(cf_ctx* c, int block) {
    const uint64_t res_bytes = c->P(block).res_bytes;
    if (!res_bytes || !c->host[block]) return CF_OK;
    if (!c->res_buf[block]) {
        if (hipMalloc((void**)&c->res_buf[block], res_bytes) != hipSuccess) {
            (void)hipGetLastError();
            return cf_fail(c, CF_ERR_NOMEM, "hipMalloc of %llu resident bytes for block %d failed",
                        (unsigned long long)res_bytes, block);
        }
    }
    CF_HIP(c, hipMemcpy(c->res_buf[block], c->host[block], res_bytes, hipMemcpyHostToDevice));
    return CF_OK;
}

inline uint64_t chunk_begin(const cf_ctx* c, int k) { return (uint64_t)k * c->chunk_bytes; }
inline uint64_t chunk_end(const cf_ctx* c, const Plan& p, int k) { return std::min(p.blob_bytes, (uint64_t)(k + 1) * c->chunk_bytes); }

WView view_of(const cf_ctx* c, int block) {
    WView v;
    v.lo = (const char*)c->res_buf[block];
    const int sl = c->block_slot[block];
    v.hi = (sl >= 0 && c->slot[sl]) ? (const char*)c->slot[sl] - c->P(block).res_bytes : nullptr;
    v.split = c->P(block).res_bytes;
    return v;
}

// ------------------------------------------------------------------------------------------
// prefetch worker (Sec. 3.2): enqueues chunk copies with at most pause_depth (1 or 2) in flight and, when
// the compute stream has reached a collective, parks the copy stream on that collective's completion event
// ------------------------------------------------------------------------------------------
// Collectives that have finished leave the list and hand their events back.  Called with c->mu held.
void retire_finished_collectives(cf_ctx* c) {
    while (!c->comm_pending.empty()) {
        PendingComm& p = c->comm_pending.front();
        if (!p.done_recorded || hipEventQuery(p.done) != hipSuccess) break;
        c->comm_ev_pool.push_back(p.ready);
        c->comm_ev_pool.push_back(p.done);
        c->comm_pending.pop_front();
    }
    (void)hipGetLastError();                          // hipErrorNotReady of a query is not an error
}

// Pause decision of the prefetch worker, taken before each chunk copy is enqueued (Sec. 3.2: the flag is
// checked at chunk boundaries).  A collective counts as issued once the compute stream has reached it in
// GPU time (its `ready` event has fired), not when the host enqueued it: the host runs a block ahead of the
// GPU.  The copy stream is then parked on the collective's completion event, once per collective; the chunk
// already on the link finishes first, which is the residual stall the paper bounds by one chunk's service
// time (with pause_depth = 1 no further chunk is queued behind it).  Called with c->mu held.
int pause_if_collective_running(cf_ctx* c, hipStream_t copy, std::unique_lock<std::mutex>& lk) {
    retire_finished_collectives(c);
    if (c->comm_pending.empty()) return CF_OK;
    PendingComm& p = c->comm_pending.front();
    if (p.handled || hipEventQuery(p.ready) != hipSuccess) { (void)hipGetLastError(); return CF_OK; }
    // the caller is between cf_comm_begin and cf_comm_end: its completion event is recorded within microseconds
    c->cv.wait_for(lk, std::chrono::milliseconds(200), [&] { return c->comm_pending.front().done_recorded || c->worker_stop; });
    PendingComm& q = c->comm_pending.front();
    if (!q.done_recorded) return CF_OK;               // cf_comm_end never came: nothing to wait for
    CF_HIP(c, hipStreamWaitEvent(copy, q.done, 0));
    q.handled = true;
    c->stats.pauses++;
    return CF_OK;
}

int enqueue_block_copies(cf_ctx* c, int block, int s, hipStream_t copy, bool bounded) {
    const Plan& p = c->P(block);
    if (c->done_valid[s]) CF_HIP(c, hipStreamWaitEvent(copy, c->done_ev[s], 0));   // slot's last reader
    for (int k = p.n_res_chunks; k < p.n_chunks; ++k) {
        if (bounded) {
            const int depth = c->pause_depth;
            if (k - depth >= p.n_res_chunks) CF_HIP(c, hipEventSynchronize(c->chunk_ev[s][k - depth]));
            std::unique_lock<std::mutex> lk(c->mu);
            CF_TRY(pause_if_collective_running(c, copy, lk));
        }
        const uint64_t b = chunk_begin(c, k), e = chunk_end(c, p, k);
        CF_HIP(c, hipMemcpyAsync(c->slot[s] + (b - p.res_bytes), c->host[block] + b, e - b, hipMemcpyHostToDevice, copy));
        CF_HIP(c, hipEventRecord(c->chunk_ev[s][k], copy));
        {
            std::lock_guard<std::mutex> lk(c->mu);
            c->enq_count[s] = k + 1;
            c->stats.h2d_bytes += e - b;
            c->stats.h2d_chunks++;
        }
        c->cv.notify_all();
    }
    CF_HIP(c, hipEventRecord(c->land_ev[s], copy));
    c->land_valid[s] = true;
    return CF_OK;
}

void worker_main(cf_ctx* c) {
    (void)hipSetDevice(c->device);
    std::string my_err;
    t_err_sink = &my_err;
    for (;;) {
        PrefetchJob job;
        {
            std::unique_lock<std::mutex> lk(c->mu);
            c->cv.wait(lk, [&] { return c->worker_stop || !c->jobs.empty(); });
            if (c->jobs.empty()) return;
            job = c->jobs.front();
            c->jobs.pop_front();
            c->worker_busy = true;
        }
        int rc = enqueue_block_copies(c, job.block, job.slot, job.copy, true);
        {
            std::lock_guard<std::mutex> lk(c->mu);
            if (rc != CF_OK) {
                c->worker_err = my_err;
                c->enq_count[job.slot] = c->max_chunks;   // never leave the consumer waiting
            }
            c->worker_busy = false;
        }
        c->cv.notify_all();
    }
}

void worker_drain(cf_ctx* c) {
    if (!c->worker.joinable()) return;
    std::unique_lock<std::mutex> lk(c->mu);
    c->cv.wait(lk, [&] { return c->jobs.empty() && !c->worker_busy; });
}

void worker_stop(cf_ctx* c) {
    if (!c->worker.joinable()) return;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        c->worker_stop = true;
    }
    c->cv.notify_all();
    c->worker.join();
    c->worker_stop = false;
}

// ------------------------------------------------------------------------------------------
// profiling: hipEvent pair around each kernel launch, resolved lazily
// ------------------------------------------------------------------------------------------
enum Kid {
    K_MODVEC, K_LN, K_LIN1, K_QKV, K_RELAYOUT, K_ATTN, K_LIN2, K_OUT, K_UP, K_DOWN,
    K_CROSS_Q, K_CROSS_KV, K_CROSS_ATTN, K_CROSS_OUT,
    // not kernels: time the compute stream spends parked on a chunk's event (the exposed prefetch of
    // Sec. 4.3's breakdown) and on an emulated collective's completion
    K_CHUNK_WAIT, K_COMM_WAIT, K_COUNT
};
const char* kKidName[K_COUNT] = {"modvec", "ln_modulate", "gemm_lin1", "gemm_qkv", "pre_attention",
                                 "attention", "gemm_lin2", "gemm_out", "gemm_up", "gemm_down",
                                 "gemm_cross_q", "gemm_cross_kv", "cross_attention", "gemm_cross_out",
                                 "prefetch_stall", "collective_wait"};

hipEvent_t prof_event(cf_ctx* c) {
    if (!c->ev_pool.empty()) { hipEvent_t e = c->ev_pool.back(); c->ev_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}

// kid + K_COUNT * variant; variant = the GEMM's tile shape (gemm_tile)
struct ProfScope {
    cf_ctx* c; hipStream_t s; ProfEntry pe; bool on;
    ProfScope(cf_ctx* c_, hipStream_t s_, int kid, double flops, double bytes, int variant = 0)
        : c(c_), s(s_), on(c_->profiling) {
        if (!on) return;
        pe = ProfEntry{kid + K_COUNT * variant, prof_event(c), prof_event(c), flops, bytes};
        (void)hipEventRecord(pe.a, s);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(pe.b, s);
        c->prof_pending.push_back(pe);
    }
};

int prof_resolve(cf_ctx* c) {
    if (c->prof_pending.empty()) return CF_OK;
    CF_HIP(c, hipDeviceSynchronize());
    if (c->ktimes.empty()) {
        c->ktimes.resize(2 * K_COUNT);
        for (int i = 0; i < 2 * K_COUNT; ++i) {
            memset(&c->ktimes[i], 0, sizeof(cf_kernel_time));
            const bool gemm = strncmp(kKidName[i % K_COUNT], "gemm_", 5) == 0;
            snprintf(c->ktimes[i].name, sizeof c->ktimes[i].name, "%s%s", kKidName[i % K_COUNT],
                     gemm ? (i < K_COUNT ? "/256x256" : "/128x128") : "");
        }
    }
    for (auto& pe : c->prof_pending) {
        float ms = 0.f;
        CF_HIP(c, hipEventElapsedTime(&ms, pe.a, pe.b));
        cf_kernel_time& k = c->ktimes[pe.kid];
        k.launches++;
        k.total_ms += ms;
        k.flops += pe.flops;
        k.bytes += pe.bytes;
        c->ev_pool.push_back(pe.a);
        c->ev_pool.push_back(pe.b);
    }
    c->prof_pending.clear();
    return CF_OK;
}

// device-side wait for chunk k of `block` on stream s
int wait_chunk(cf_ctx* c, int block, int k, hipStream_t s) {
    if (k < c->P(block).n_res_chunks) return CF_OK;
    const int sl = c->block_slot[block];
    if (sl < 0 || c->slot_tenant[sl] != block || c->slot_state[sl] == SLOT_EMPTY)
        return cf_fail(c, CF_ERR_STATE, "block %d: chunk %d awaited but its prefetch was not begun", block, k);
    if (c->worker.joinable()) {
        std::unique_lock<std::mutex> lk(c->mu);
        c->cv.wait(lk, [&] { return c->enq_count[sl] > k; });
        if (!c->worker_err.empty()) return cf_fail(c, CF_ERR_HIP, "prefetch worker: %s", c->worker_err.c_str());
    }
    ProfScope ps(c, s, K_CHUNK_WAIT, 0, 0);
    CF_HIP(c, hipStreamWaitEvent(s, c->chunk_ev[sl][k], 0));
    return CF_OK;
}


// ------------------------------------------------------------------------------------------
// forward building blocks
// ------------------------------------------------------------------------------------------
struct Fwd {
    cf_ctx* c;
    int block;
    hipStream_t s;
    WView W;
    const cf_block_io* io;
    Ws ws;
};

const TensorDesc& T(const Fwd& F, const std::string& name) {
    for (auto& t : F.c->P(F.block).tensors)
        if (t.name == name) return t;
    static TensorDesc none{"", 0, 0, 0};
    return none;
}

// wait for every chunk a (small) tensor touches
int need(Fwd& F, const TensorDesc& t) {
    // the copy stream is in order: the last chunk's event covers the earlier ones
    const int last = (int)((t.off + t.bytes() - 1) / F.c->chunk_bytes);
    if (last >= F.c->P(F.block).n_res_chunks && last > F.c->waited_upto) {
        CF_TRY(wait_chunk(F.c, F.block, last, F.s));
        F.c->waited_upto = last;
    }
    return CF_OK;
}

// Panel plan of a weight matrix (pure host arithmetic): rows become usable chunk by chunk, so the
// matrix is cut into panels [row0, row1), each tagged with the last chunk that must have landed
// before it may run (-1: needs no streamed chunk beyond `already`).  Before blocking on a chunk
// that is still streaming, rows whose bytes lie in earlier chunks form a panel.  `already` =
// highest chunk known to be present (resident prefix or waited for earlier).
//
// How many of the usable rows go into the panel: every launch ends with a partly filled round of
// workgroups, and a layer cut at arbitrary rows pays that once per panel (measured on the video
// shares: three panels made the MLP-in layer 14 % slower than one launch).  For a linear layer
// over m_rows tokens the panel is the largest number of whole 256-feature tiles whose launch fills
// its rounds to 93 %; failing that the best-filled one if it reaches 75 %; failing that the rows
// stay with the next panel.  m_rows = 0: the modulation matrix-vector product, 8 rows at a time.
struct Panel { int row0, row1, wait; };

int panel_end(int m_rows, int row0, int avail) {
    if (m_rows <= 0) return std::max(row0, avail / 8 * 8);
    int best = 0;
    double best_fill = 0;
    for (int f = (avail - row0) / 256; f >= 1; --f) {
        const double fill = gemm_fill(m_rows, 256 * f);
        if (fill >= 0.93) return row0 + 256 * f;
        if (fill > best_fill) best_fill = fill, best = f;
    }
    return best_fill >= 0.75 ? row0 + 256 * best : row0;
}

std::vector<Panel> plan_panels(const cf_ctx* c, const TensorDesc& t, int m_rows, int already) {
    std::vector<Panel> out;
    const uint64_t row_bytes = 2ull * t.cols;
    const int first = (int)(t.off / c->chunk_bytes), last = (int)((t.off + t.bytes() - 1) / c->chunk_bytes);
    int row0 = 0, pending_wait = -1;
    for (int k = first; k <= last; ++k) {
        if (k <= already) continue;
        const uint64_t lim = chunk_begin(c, k);
        const int avail = lim <= t.off ? 0 : (int)std::min<uint64_t>(t.rows, (lim - t.off) / row_bytes);
        const int end = avail > row0 ? panel_end(m_rows, row0, avail) : row0;
        if (end > row0) {
            out.push_back(Panel{row0, end, pending_wait});
            row0 = end;
        }
        pending_wait = k;               // rows beyond `avail` need chunk k
    }
    if ((int)t.rows > row0) out.push_back(Panel{row0, (int)t.rows, pending_wait});
    return out;
}

// Launch `fn(row0, row1)` over the panels of weight matrix t, each behind its chunk wait.
template <class Fn>
int panels(Fwd& F, const TensorDesc& t, int m_rows, Fn&& fn) {
    cf_ctx* c = F.c;
    const int n_res = c->P(F.block).n_res_chunks;
    for (const Panel& p : plan_panels(c, t, m_rows, std::max(c->waited_upto, n_res - 1))) {
        if (p.wait > c->waited_upto && p.wait >= n_res) {
            CF_TRY(wait_chunk(c, F.block, p.wait, F.s));
            c->waited_upto = p.wait;
        }
        CF_TRY(fn(p.row0, p.row1));
    }
    return CF_OK;
}

// modulation vectors of every sample: t is [batch, d], out + b*out_bs receives sample b's
int run_modvec(Fwd& F, const std::string& wname, const std::string& bname, const float* t, float* out, long out_bs) {
    const TensorDesc &w = T(F, wname), &b = T(F, bname);
    CF_TRY(need(F, b));
    const int B = batch_of(F.c->d);
    return panels(F, w, 0, [&](int r0, int r1) -> int {
        ProfScope ps(F.c, F.s, K_MODVEC, 2.0 * B * (r1 - r0) * w.cols, 2.0 * (r1 - r0) * w.cols);
        CF_HIP(F.c, modvec_launch(F.W, w.off, b.off, t, out, r0, r1, (int)w.cols, B, out_bs, F.s));
        return CF_OK;
    });
}

// `rows` rows of the whole batch, rows_per_sample of them per sample (0: one sample); sample b is read at
// x + b*x_bs and modulated with shift + b*mod_bs, scale + b*mod_bs
int run_ln_mod(Fwd& F, const float* x, const float* shift, const float* scale, bf16* out, int rows, int rows_per_sample,
               long x_bs, long mod_bs) {
    if (rows <= 0) return CF_OK;
    ProfScope ps(F.c, F.s, K_LN, 0, 6.0 * rows * F.c->d.d);
    CF_HIP(F.c, ln_modulate_launch(x, shift, scale, out, rows, F.c->d.d, F.c->d.d, rows_per_sample, x_bs, mod_bs, F.s));
    return CF_OK;
}

// out-feature panels of one linear layer; `g` carries everything but the panel and the weights
int run_linear(Fwd& F, int kid, const std::string& wname, const std::string& bname, GemmArgs g) {
    if (g.M <= 0) return CF_OK;
    const TensorDesc &w = T(F, wname), &b = T(F, bname);
    CF_TRY(need(F, b));
    g.W = F.W;
    g.act_erf = F.c->d.gelu_erf;
    g.w_off = w.off;
    g.bias_off = b.off;
    g.has_bias = 1;
    g.N = (int)w.rows;
    g.K = (int)w.cols;
    if (g.epi == EPI_SPLIT_GELU && g.n_split > g.N) g.n_split = g.N;
    return panels(F, w, g.M, [&](int r0, int r1) -> int {
        GemmArgs p = g;
        p.n0 = r0;
        p.n1 = r1;
        if (const char* msg = gemm_check(p)) return cf_fail(F.c, CF_ERR_ARG, "%s (%s)", msg, wname.c_str());
        ProfScope ps(F.c, F.s, kid, 2.0 * p.M * (r1 - r0) * p.K, 0, gemm_tile(p));
        CF_HIP(F.c, gemm_launch(p, F.s));
        return CF_OK;
    });
}

// Two independent linear layers (the two streams of a double-stream block; the query and the context
// projections of a cross-attention).  When neither needs a chunk that has not been waited for yet they
// go out as one launch, so that the small one's few workgroups ride along with the large one's instead
// of holding the chip for the length of their K loop; otherwise (weights still streaming) each takes
// its own panel launches as usual.
int run_linear_pair(Fwd& F, int kid, const std::string (&wname)[2], const std::string (&bname)[2], const GemmArgs (&g_in)[2]) {
    cf_ctx* c = F.c;
    const int have = std::max(c->waited_upto, c->P(F.block).n_res_chunks - 1);
    bool pair = g_in[0].M > 0 && g_in[1].M > 0;
    GemmArgs g[2];
    for (int i = 0; i < 2 && pair; ++i) {
        const TensorDesc &w = T(F, wname[i]), &b = T(F, bname[i]);
        const int last = (int)((std::max(w.off + w.bytes(), b.off + b.bytes()) - 1) / c->chunk_bytes);
        if (last > have) pair = false;
        g[i] = g_in[i];
        g[i].W = F.W;
        g[i].act_erf = c->d.gelu_erf;
        g[i].w_off = w.off;
        g[i].bias_off = b.off;
        g[i].has_bias = 1;
        g[i].N = (int)w.rows;
        g[i].K = (int)w.cols;
        g[i].n0 = 0;
        g[i].n1 = g[i].N;
        if (g[i].epi == EPI_SPLIT_GELU && g[i].n_split > g[i].N) g[i].n_split = g[i].N;
    }
    const int tile = pair ? gemm_pair_tile(g[0], g[1]) : -1;
    if (tile < 0) {
        CF_TRY(run_linear(F, kid, wname[0], bname[0], g_in[0]));
        return run_linear(F, kid, wname[1], bname[1], g_in[1]);
    }
    for (int i = 0; i < 2; ++i)
        if (const char* msg = gemm_check(g[i])) return cf_fail(c, CF_ERR_ARG, "%s (%s)", msg, wname[i].c_str());
    ProfScope ps(c, F.s, kid, 2.0 * g[0].M * g[0].N * g[0].K + 2.0 * g[1].M * g[1].N * g[1].K, 0, tile);
    CF_HIP(c, gemm_launch_pair(g[0], g[1], F.s));
    return CF_OK;
}

TokenMap token_map(const cf_model_desc& m) {
    TokenMap t;
    t.n_total = m.n_total;
    t.n_local = m.n_total / m.sp_degree;
    if (m.n_txt_total > 0) {            // text rows, then image rows, each split contiguously over the ranks
        const int tl = m.n_txt_total / m.sp_degree, il = t.n_local - tl;
        t.pos0 = m.sp_rank * tl; t.len0 = tl;
        t.pos1 = m.n_txt_total + m.sp_rank * il; t.len1 = il;
    } else {
        t.pos0 = m.sp_rank * t.n_local; t.len0 = t.n_local;
        t.pos1 = m.n_total; t.len1 = 0;
    }
    return t;
}

// emulated collectives standing for the Ulysses exchanges (n of them back to back)
int cf_comm_begin_impl(cf_ctx* c, hipStream_t comm, hipStream_t compute);
int cf_comm_end_impl(cf_ctx* c, hipStream_t comm, hipStream_t compute);

int emulate_collectives(Fwd& F, int n) {
    cf_ctx* c = F.c;
    if (!c->comm_stream || !c->comm_bytes) return CF_OK;
    CF_TRY(cf_comm_begin_impl(c, c->comm_stream, F.s));
    const uint64_t half = c->comm_bytes / 2;
    for (int i = 0; i < n; ++i) {
        CF_HIP(c, hipMemcpyAsync(c->comm_dev, c->comm_host, half, hipMemcpyHostToDevice, c->comm_stream));
        CF_HIP(c, hipMemcpyAsync(c->comm_host + half, c->comm_dev + half, half, hipMemcpyDeviceToHost, c->comm_stream));
        c->stats.comm_bytes_h2d += half;
        c->stats.comm_bytes_d2h += half;
    }
    return cf_comm_end_impl(c, c->comm_stream, F.s);
}

// Where the attention rows of the local tokens go (operand of the output projection): sample b's rows
// of the map's first segment at dst + b*bs0, of the second at dst1 + b*bs1 (dst1 NULL: they follow the
// first segment, bs0 then spans the whole sample); leading dimension ld.
struct AttnOut {
    bf16* dst; bf16* dst1; int ld; long bs0, bs1;
};

// q/k/v of the local rows (already in ws.qkv) -> attention over the joint sequence -> rows of all
// heads for the local tokens.  `parts` describe sample 0; sample b's rows follow densely
// (b * rows * ld further), its operands and peer/send buffers one sample further each.
int run_joint_attention(Fwd& F, const RelayoutArgs* parts, int n_parts, const AttnOut& out) {
    cf_ctx* c = F.c;
    const cf_model_desc& m = c->d;
    const int P = m.sp_degree, hl = m.n_heads / P, h0 = m.sp_rank * hl, hd = m.head_dim, B = batch_of(m);
    const TokenMap map = token_map(m);
    const int npad = n_pad_of(m.n_total);
    const size_t n_rem = (size_t)(map.n_total - map.n_local);
    const cf_block_io* io = F.io;
    if (P > 1 && (!io->peer_q || !io->peer_k || !io->peer_v || !io->peer_attn))
        return cf_fail(c, CF_ERR_ARG, "sp_degree > 1 needs peer_q, peer_k, peer_v and peer_attn");
    const size_t op_bs = (size_t)hl * m.n_total * hd, vt_bs = (size_t)hl * hd * npad;        // Q,K / Vt per sample
    const size_t peer_bs = (size_t)hl * n_rem * hd, send_bs = (size_t)(m.n_heads - hl) * map.n_local * hd;
    const bool direct = P == 1 && !out.dst1;        // attention writes the projection operand row by row itself
    const size_t pa_bs = (size_t)map.n_local * (m.n_heads - hl) * hd;
    for (int b = 0; b < B; ++b) {
        RelayoutArgs pb[2];
        double bytes = 0;
        for (int i = 0; i < n_parts; ++i) {
            RelayoutArgs& r = pb[i];
            r = parts[i];
            r.src += (size_t)b * r.rows * r.ld;
            r.Q += b * op_bs; r.K += b * op_bs; r.Vt += b * vt_bs;
            if (r.send_q) r.send_q += b * send_bs;
            if (r.send_k) r.send_k += b * send_bs;
            if (r.send_v) r.send_v += b * send_bs;
            bytes += 2.0 * 2 * r.rows * 3.0 * m.d;
        }
        // what the second exchange delivers (the other heads' attention rows of the local tokens) is an input
        // of the block: it is put in place by the same launch, ahead of attention
        PeerAttnArgs pa{};
        if (P > 1) {
            bytes += 2.0 * 2 * 3 * hl * (double)n_rem * hd + 2.0 * 2 * (double)pa_bs;
            pa.peer_attn = (const bf16*)io->peer_attn + b * pa_bs;
            pa.dst = out.dst + b * out.bs0;
            pa.dst1 = out.dst1 ? out.dst1 + b * out.bs1 : nullptr;
            pa.ld = out.ld; pa.n_heads = m.n_heads; pa.h0 = h0; pa.h_local = hl; pa.hd = hd; pa.map = map;
        }
        ProfScope ps(c, F.s, K_RELAYOUT, 0, bytes);
        CF_HIP(c, pre_attention_launch(pb, n_parts, P > 1 ? (const bf16*)io->peer_q + b * peer_bs : nullptr,
                                       P > 1 ? (const bf16*)io->peer_k + b * peer_bs : nullptr,
                                       P > 1 ? (const bf16*)io->peer_v + b * peer_bs : nullptr, pa, F.s));
    }
    CF_TRY(emulate_collectives(F, 3));
    AttnArgs a{};
    a.Q = F.ws.Q; a.K = F.ws.K; a.Vt = F.ws.Vt;
    a.H = B * hl; a.hps = hl; a.nq = m.n_total; a.nk = m.n_total; a.nk_pad = npad; a.hd = hd;
    a.scale = 1.0f / sqrtf((float)hd);
    if (direct) {
        a.O = out.dst; a.o_hs = hd; a.o_qs = out.ld; a.o_bs = out.bs0;
    } else {
        // the attention kernel's stores do the second exchange: rows of this rank's positions go to the
        // projection operand, the others to the send buffer
        a.scatter = 1;
        a.map = map;
        a.dst0 = out.dst; a.bs0 = out.bs0;
        a.dst1 = out.dst1 ? out.dst1 : out.dst + (size_t)map.len0 * out.ld;
        a.bs1 = out.dst1 ? out.bs1 : out.bs0;
        a.ld = out.ld; a.h0 = h0;
        a.send = (bf16*)io->send_attn; a.send_bs = (long)peer_bs;
    }
    if (const char* msg = attn_check(a)) return cf_fail(c, CF_ERR_ARG, "%s", msg);
    {
        ProfScope ps(c, F.s, K_ATTN, 4.0 * B * hl * (double)m.n_total * m.n_total * hd, 0);
        CF_HIP(c, attn_launch(a, F.s));
    }
    return emulate_collectives(F, 1);
}

RelayoutArgs relayout_for(Fwd& F, const bf16* src, int rows, int row0, const std::string& qn, const std::string& kn) {
    const cf_model_desc& m = F.c->d;
    RelayoutArgs r{};
    r.src = src; r.ld = 3 * m.d; r.rows = rows;
    r.col_q = 0; r.col_k = m.d; r.col_v = 2 * m.d;
    r.n_heads = m.n_heads;
    r.h_local = m.n_heads / m.sp_degree;
    r.h0 = m.sp_rank * r.h_local;
    r.hd = m.head_dim;
    r.W = F.W;
    r.has_norm = m.qk_rmsnorm;
    if (m.qk_rmsnorm) { r.qn_off = T(F, qn).off; r.kn_off = T(F, kn).off; }
    r.map = token_map(m);
    r.row0 = row0;
    r.Q = F.ws.Q; r.K = F.ws.K; r.Vt = F.ws.Vt;
    r.n_pad = n_pad_of(m.n_total);
    r.send_q = (bf16*)F.io->send_q; r.send_k = (bf16*)F.io->send_k; r.send_v = (bf16*)F.io->send_v;
    r.rope_cos = F.io->rope_cos; r.rope_sin = F.io->rope_sin;
    return r;
}

// sample strides of the caller's residual streams (elements); 0 in the io struct = dense
long x_stride(const cf_block_io* io, long dense) { return io->x_sample_stride ? (long)io->x_sample_stride : dense; }
long x_txt_stride(const cf_block_io* io, long dense) { return io->x_txt_sample_stride ? (long)io->x_txt_sample_stride : dense; }

// batch bookkeeping of a residual epilogue: rows per sample and the sample strides of gate, resid, y
GemmArgs batched(GemmArgs g, int batch, int rows_per_sample, long gate_bs, long resid_bs, long y_bs) {
    if (batch > 1) { g.rows_per_sample = rows_per_sample; g.gate_bs = gate_bs; g.resid_bs = resid_bs; g.y_bs = y_bs; }
    return g;
}

// ---- MM-DiT single-stream block (App. B)
int fwd_single(Fwd& F) {
    cf_ctx* c = F.c;
    const cf_model_desc& m = c->d;
    const int d = m.d, f = m.f, nl = m.n_total / m.sp_degree, B = batch_of(m), rows = B * nl, rps = B > 1 ? nl : 0;
    const cf_block_io* io = F.io;
    const long mod_bs = 3L * d, xs = x_stride(io, (long)nl * d);
    CF_TRY(run_modvec(F, "w_mod", "b_mod", io->temb, F.ws.mod, mod_bs));
    const float *shift = F.ws.mod, *scale = F.ws.mod + d, *gate = F.ws.mod + 2 * d;
    CF_TRY(run_ln_mod(F, io->x, shift, scale, F.ws.xn, rows, rps, xs, mod_bs));
    if (m.qk_rmsnorm) { CF_TRY(need(F, T(F, "q_norm"))); CF_TRY(need(F, T(F, "k_norm"))); }
    GemmArgs g{};
    g.A = F.ws.xn; g.lda = d; g.M = rows; g.epi = EPI_SPLIT_GELU;
    g.out0 = F.ws.qkv; g.ld0 = 3 * d; g.n_split = 3 * d;
    g.out1 = F.ws.c; g.ld1 = d + f; g.col1_off = d;
    CF_TRY(run_linear(F, K_LIN1, "w1", "b1", g));
    RelayoutArgs r = relayout_for(F, F.ws.qkv, nl, 0, "q_norm", "k_norm");
    CF_TRY(run_joint_attention(F, &r, 1, AttnOut{F.ws.c, nullptr, d + f, (long)nl * (d + f), 0}));
    GemmArgs h{};
    h.A = F.ws.c; h.lda = d + f; h.M = rows; h.epi = EPI_GATE_RESID;
    h.resid = io->x; h.gate = gate; h.y = io->y; h.ldy = d;
    return run_linear(F, K_LIN2, "w2", "b2", batched(h, B, nl, mod_bs, xs, xs));
}

int fwd_dit(Fwd& F);
int fwd_double(Fwd& F);

int check_desc(const cf_model_desc* m) {
    if (!m) return cf_fail(nullptr, CF_ERR_ARG, "null description");
    if (m->kind < 0 || m->kind > 2) return cf_fail(nullptr, CF_ERR_ARG, "unknown block kind %d", m->kind);
    if (m->n_blocks <= 0) return cf_fail(nullptr, CF_ERR_ARG, "n_blocks must be positive");
    if (m->head_dim != 64 && m->head_dim != 128) return cf_fail(nullptr, CF_ERR_ARG, "head_dim must be 64 or 128");
    if (m->n_heads <= 0 || m->d != m->n_heads * m->head_dim) return cf_fail(nullptr, CF_ERR_ARG, "d must equal n_heads * head_dim");
    if (m->d % 256 || m->d > 4096) return cf_fail(nullptr, CF_ERR_ARG, "d must be a multiple of 256, at most 4096");
    const int nj = m->d / 256;
    if (!(nj == 1 || nj == 2 || nj == 3 || nj == 4 || nj == 6 || nj == 8 || nj == 12 || nj == 16))
        return cf_fail(nullptr, CF_ERR_ARG, "d/256 must be one of 1,2,3,4,6,8,12,16");
    if (m->f <= 0 || m->f % 64) return cf_fail(nullptr, CF_ERR_ARG, "f must be a positive multiple of 64");
    if (m->sp_degree <= 0 || m->sp_rank < 0 || m->sp_rank >= m->sp_degree) return cf_fail(nullptr, CF_ERR_ARG, "bad sp_degree/sp_rank");
    if (m->n_heads % m->sp_degree) return cf_fail(nullptr, CF_ERR_ARG, "sp_degree must divide n_heads");
    if (m->n_total <= 0 || m->n_total % m->sp_degree) return cf_fail(nullptr, CF_ERR_ARG, "sp_degree must divide n_total");
    if (m->kind == CF_DOUBLE_STREAM && m->n_txt_total <= 0) return cf_fail(nullptr, CF_ERR_ARG, "double-stream needs n_txt_total > 0");
    if (m->n_txt_total) {
        if (m->kind == CF_DIT_CROSS) return cf_fail(nullptr, CF_ERR_ARG, "n_txt_total has no meaning for DiT blocks");
        if (m->n_txt_total < 0 || m->n_txt_total >= m->n_total || m->n_txt_total % m->sp_degree)
            return cf_fail(nullptr, CF_ERR_ARG, "need 0 < n_txt_total < n_total, divisible by sp_degree");
    }
    if (m->kind == CF_DIT_CROSS && m->l_ctx <= 0) return cf_fail(nullptr, CF_ERR_ARG, "DiT block needs l_ctx > 0");
    if (m->gelu_erf != 0 && m->gelu_erf != 1) return cf_fail(nullptr, CF_ERR_ARG, "gelu_erf must be 0 or 1");
    if (m->batch < 0 || m->batch > 1024) return cf_fail(nullptr, CF_ERR_ARG, "batch must be in [0, 1024] (0 = 1)");
    if ((int64_t)std::max(1, m->batch) * (m->n_total / m->sp_degree) > (1 << 30)) return cf_fail(nullptr, CF_ERR_ARG, "batch * n_local too large");
    if (m->chunk_bytes == 0 || m->chunk_bytes % 256) return cf_fail(nullptr, CF_ERR_ARG, "chunk_bytes must be a positive multiple of 256");
    return CF_OK;
}

// (re)build the plans of the kinds the model uses
void plan_model(cf_ctx* c) {
    for (int k = 0; k < 3; ++k) c->plan[k] = Plan{};
    c->ws_bytes = 0;
    c->max_chunks = 0;
    for (int k : c->block_kind) {
        Plan& p = c->plan[k];
        if (p.kind >= 0) continue;
        plan_layout(&p, c->d, k, c->chunk_bytes);
        p.ws_bytes = carve(c->d, k, nullptr).total;
        c->ws_bytes = std::max(c->ws_bytes, p.ws_bytes);
        c->max_chunks = std::max(c->max_chunks, p.n_chunks);
    }
}

// A prefetch counts as hidden when its last chunk landed at least this long before the block that ran ahead of
// its consumer ended: a margin of a few event-timestamp granules (timestamps of two streams are only comparable
// to some microseconds), small against any block that could hide a prefetch at all.
constexpr float kLandedAheadMs = 0.05f;

int check_block(const cf_ctx* c, int block) {
    if (!c) return CF_ERR_ARG;
    if (block < 0 || block >= c->d.n_blocks) return cf_fail(c, CF_ERR_ARG, "block %d out of range [0,%d)", block, c->d.n_blocks);
    return CF_OK;
}

}  // namespace

// ==========================================================================================
// ABI
// ==========================================================================================
extern "C" {

int cf_create(const cf_model_desc* desc, cf_ctx** out) {
    if (!out) return cf_fail(nullptr, CF_ERR_ARG, "null out pointer");
    *out = nullptr;
    CF_TRY(check_desc(desc));
    cf_ctx* c = new (std::nothrow) cf_ctx();
    if (!c) return cf_fail(nullptr, CF_ERR_NOMEM, "out of host memory");
    c->d = *desc;
    c->chunk_bytes = desc->chunk_bytes;
    c->block_kind.assign(desc->n_blocks, desc->kind);
    plan_model(c);
    c->host.assign(desc->n_blocks, nullptr);
    c->res_buf.assign(desc->n_blocks, nullptr);
    c->block_slot.assign(desc->n_blocks, -1);
    *out = c;
    return CF_OK;
}

int cf_destroy(cf_ctx* c) {
    if (!c) return CF_ERR_ARG;
    worker_drain(c);
    worker_stop(c);
    if (c->device_ready) {
        (void)hipDeviceSynchronize();
        free_weights(c);
        for (int s = 0; s < 2; ++s) {
            for (auto e : c->chunk_ev[s]) (void)hipEventDestroy(e);
            (void)hipEventDestroy(c->done_ev[s]);
            (void)hipEventDestroy(c->land_ev[s]);
        }
        (void)hipEventDestroy(c->comm_ready_ev);
        (void)hipEventDestroy(c->comm_done_ev);
        for (auto e : c->fwd_ev) (void)hipEventDestroy(e);
        for (auto& pc : c->comm_pending) { (void)hipEventDestroy(pc.ready); (void)hipEventDestroy(pc.done); }
        for (auto e : c->comm_ev_pool) (void)hipEventDestroy(e);
        for (auto& pe : c->prof_pending) { (void)hipEventDestroy(pe.a); (void)hipEventDestroy(pe.b); }
        for (auto e : c->ev_pool) (void)hipEventDestroy(e);
        if (c->comm_dev) (void)hipFree(c->comm_dev);
        if (c->checksum_dev) (void)hipFree(c->checksum_dev);
    }
    delete c;
    return CF_OK;
}

const char* cf_last_error(const cf_ctx* c) { return c ? c->err.c_str() : g_create_err.c_str(); }

int cf_set_block_kinds(cf_ctx* c, const int32_t* kinds, int32_t n) {
    if (!c || !kinds) return CF_ERR_ARG;
    if (n != c->d.n_blocks) return cf_fail(c, CF_ERR_ARG, "%d kinds given for %d blocks", n, c->d.n_blocks);
    if (c->device_ready) return cf_fail(c, CF_ERR_STATE, "block kinds must be set before any block is registered");
    for (int b = 0; b < n; ++b) {
        if (kinds[b] < 0 || kinds[b] > 2) return cf_fail(c, CF_ERR_ARG, "block %d: unknown kind %d", b, kinds[b]);
        if (kinds[b] == CF_DOUBLE_STREAM && c->d.n_txt_total <= 0) return cf_fail(c, CF_ERR_ARG, "block %d: double-stream needs n_txt_total > 0", b);
        if (kinds[b] == CF_DIT_CROSS && (c->d.l_ctx <= 0 || c->d.n_txt_total)) return cf_fail(c, CF_ERR_ARG, "block %d: DiT block needs l_ctx > 0 and no text rows", b);
    }
    c->block_kind.assign(kinds, kinds + n);
    plan_model(c);
    return CF_OK;
}

int cf_block_kind_of(const cf_ctx* c, int32_t block, int32_t* out) {
    CF_TRY(check_block(c, block));
    if (!out) return CF_ERR_ARG;
    *out = c->block_kind[block];
    return CF_OK;
}

int cf_blob_bytes_of(const cf_ctx* c, int32_t block, uint64_t* out) {
    CF_TRY(check_block(c, block));
    if (!out) return CF_ERR_ARG;
    *out = c->P(block).blob_bytes;
    return CF_OK;
}

int cf_n_chunks_of(const cf_ctx* c, int32_t block, int32_t* out) {
    CF_TRY(check_block(c, block));
    if (!out) return CF_ERR_ARG;
    *out = c->P(block).n_chunks;
    return CF_OK;
}

int cf_blob_layout_of(const cf_ctx* c, int32_t block, cf_tensor_slot* out, int32_t* n) {
    CF_TRY(check_block(c, block));
    if (!n) return CF_ERR_ARG;
    const std::vector<TensorDesc>& ts = c->P(block).tensors;
    const int cnt = (int)ts.size();
    if (out) {
        if (*n < cnt) return cf_fail(c, CF_ERR_ARG, "layout needs room for %d tensors", cnt);
        for (int i = 0; i < cnt; ++i) {
            memset(&out[i], 0, sizeof out[i]);
            snprintf(out[i].name, sizeof out[i].name, "%s", ts[i].name.c_str());
            out[i].offset = ts[i].off;
            out[i].rows = ts[i].rows;
            out[i].cols = ts[i].cols;
        }
    }
    *n = cnt;
    return CF_OK;
}

int cf_blob_bytes(const cf_ctx* c, uint64_t* out) { return cf_blob_bytes_of(c, 0, out); }
int cf_n_chunks(const cf_ctx* c, int32_t* out) { return cf_n_chunks_of(c, 0, out); }
int cf_blob_layout(const cf_ctx* c, cf_tensor_slot* out, int32_t* n) { return cf_blob_layout_of(c, 0, out, n); }

int cf_plan_panels(const cf_ctx* c, const char* tensor, int32_t m_rows, int32_t n_resident_chunks, int32_t* row0,
                   int32_t* row1, int32_t* wait_chunk_out, int32_t* n) {
    if (!c || !tensor || !n || m_rows < 0) return CF_ERR_ARG;
    const TensorDesc* t = cf_find(c->P(0), tensor);
    if (!t) return cf_fail(c, CF_ERR_ARG, "no tensor named %s in the blob", tensor);
    if (n_resident_chunks < 0 || n_resident_chunks > c->P(0).n_chunks) return cf_fail(c, CF_ERR_ARG, "resident chunk count out of range");
    const std::vector<Panel> plan = plan_panels(c, *t, m_rows, n_resident_chunks - 1);
    if (row0 && row1 && wait_chunk_out) {
        if (*n < (int)plan.size()) return cf_fail(c, CF_ERR_ARG, "need room for %d panels", (int)plan.size());
        for (size_t i = 0; i < plan.size(); ++i) { row0[i] = plan[i].row0; row1[i] = plan[i].row1; wait_chunk_out[i] = plan[i].wait; }
    }
    *n = (int)plan.size();
    return CF_OK;
}

int cf_plan_attention(int32_t H, int32_t nq, int32_t nk, int32_t head_dim, int32_t* waves_per_workgroup) {
    if (!waves_per_workgroup || H <= 0 || nq <= 0 || nk <= 0 || (head_dim != 64 && head_dim != 128))
        return cf_fail(nullptr, CF_ERR_ARG, "cf_plan_attention: positive sizes, head_dim 64 or 128 and a result pointer are required");
    AttnArgs a{};
    a.H = H; a.nq = nq; a.nk = nk; a.hd = head_dim;
    *waves_per_workgroup = attn_waves(a);
    return CF_OK;
}

int cf_plan_linear(int32_t m_rows, int32_t n_features, int32_t* tile_rows) {
    if (!tile_rows || m_rows <= 0 || n_features <= 0)
        return cf_fail(nullptr, CF_ERR_ARG, "cf_plan_linear: positive sizes and a result pointer are required");
    GemmArgs g{};
    g.M = m_rows; g.n0 = 0; g.n1 = n_features; g.N = n_features;
    *tile_rows = gemm_tile(g) == 0 ? 256 : 128;
    return CF_OK;
}

int cf_workspace_bytes(const cf_ctx* c, uint64_t* out) {
    if (!c || !out) return CF_ERR_ARG;
    *out = c->ws_bytes;
    return CF_OK;
}

int cf_register_block(cf_ctx* c, int32_t block, const void* host_blob, uint64_t bytes) {
    CF_TRY(check_block(c, block));
    if (!host_blob) return cf_fail(c, CF_ERR_ARG, "null host blob");
    if (bytes != c->P(block).blob_bytes)
        return cf_fail(c, CF_ERR_ARG, "blob is %llu bytes, layout needs %llu", (unsigned long long)bytes, (unsigned long long)c->P(block).blob_bytes);
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, host_blob);
    if (e != hipSuccess || attr.type != hipMemoryTypeHost) {
        (void)hipGetLastError();
        return cf_fail(c, CF_ERR_ARG, "host blob must be pinned host memory (hipHostMalloc)");
    }
    CF_TRY(ensure_device(c));
    worker_drain(c);
    c->host[block] = (const uint8_t*)host_blob;
    return upload_resident(c, block);
}

int set_resident_fraction(cf_ctx* c, double r, double* actual) {
    if (!c) return CF_ERR_ARG;
    if (!(r >= 0.0 && r <= 1.0)) return cf_fail(c, CF_ERR_ARG, "resident fraction %g outside [0,1]", r);
    // per kind: the leading round(r * n_chunks) chunks; the fraction reported is over the whole model
    int n_res[3] = {0, 0, 0};
    uint64_t res_bytes[3] = {0, 0, 0}, slot_bytes = 0;
    for (int k = 0; k < 3; ++k) {
        const Plan& p = c->plan[k];
        if (p.kind < 0) continue;
        n_res[k] = (int)std::floor(r * p.n_chunks + 0.5);
        res_bytes[k] = n_res[k] ? chunk_end(c, p, n_res[k] - 1) : 0;
        slot_bytes = std::max(slot_bytes, p.blob_bytes - res_bytes[k]);
    }
    if (actual) {
        double res = 0, all = 0;
        for (int k : c->block_kind) { res += (double)res_bytes[k]; all += (double)c->plan[k].blob_bytes; }
        *actual = res / all;
    }
    CF_TRY(ensure_device(c));
    worker_drain(c);
    CF_HIP(c, hipDeviceSynchronize());
    free_weights(c);
    for (int k = 0; k < 3; ++k) { c->plan[k].n_res_chunks = n_res[k]; c->plan[k].res_bytes = res_bytes[k]; }
    for (bool& h : c->hidden_kind) h = false;                 // what was observed belonged to the old split
    if (slot_bytes) {
        for (int s = 0; s < 2; ++s)
            if (hipMalloc((void**)&c->slot[s], slot_bytes) != hipSuccess) {
                (void)hipGetLastError();
                return cf_fail(c, CF_ERR_NOMEM, "hipMalloc of a %llu-byte staging slot failed", (unsigned long long)slot_bytes);
            }
    }
    for (int b = 0; b < c->d.n_blocks; ++b) CF_TRY(upload_resident(c, b));
    return CF_OK;
}

int chunked_prefetch_begin(cf_ctx* c, int32_t block, void* copy_stream) {
    CF_TRY(check_block(c, block));
    if (!c->host[block]) return cf_fail(c, CF_ERR_STATE, "block %d has no registered host blob", block);
    CF_TRY(ensure_device(c));
    if (c->P(block).n_res_chunks == c->P(block).n_chunks) return CF_OK;   // 100 % resident: nothing to move
    if (!c->slot[0]) CF_TRY(set_resident_fraction(c, 0.0, nullptr));
    if (c->block_slot[block] >= 0 && c->slot_state[c->block_slot[block]] == SLOT_FILLED)
        return cf_fail(c, CF_ERR_STATE, "block %d is already prefetched and waiting for its forward", block);
    const int s = c->next_slot;                                    // slots alternate per prefetch
    if (c->slot_state[s] == SLOT_FILLED)
        return cf_fail(c, CF_ERR_STATE, "slot %d still holds block %d whose forward has not been issued", s, c->slot_tenant[s]);
    // Bound how far the host runs ahead of the GPU: the block that last finished in the OTHER slot
    // (two forwards back) must be done before more work is queued.  The GPU still has one whole
    // block of queued work, so it never starves, and the runtime's queues never fill up -- a host
    // that is blocked inside the runtime mid-step would leave the copy stream idle.
    if (c->done_valid[s ^ 1]) CF_HIP(c, hipEventSynchronize(c->done_ev[s ^ 1]));
    // The block that just finished (other slot) ran right before this slot's last tenant.  Had that tenant's
    // weights landed by then, its prefetch was hidden (Sec. 3.1) and blocks of its kind need one wait, not one
    // per chunk.  Evaluated before the slot's events are recorded anew.
    if (c->adaptive_waits && !c->pause_resume && c->slot_tenant[s] >= 0 && c->land_valid[s] && c->done_valid[s ^ 1] &&
        c->slot_state[s] == SLOT_CONSUMED && c->slot_fwd_seq[s ^ 1] + 1 == c->slot_fwd_seq[s]) {
        bool hidden = false;
        float ms = 0.f;
        if (hipEventQuery(c->land_ev[s]) == hipSuccess && hipEventElapsedTime(&ms, c->land_ev[s], c->done_ev[s ^ 1]) == hipSuccess)
            hidden = ms > kLandedAheadMs;
        (void)hipGetLastError();
        c->hidden_kind[c->block_kind[c->slot_tenant[s]]] = hidden;
    }
    c->next_slot ^= 1;
    if (c->slot_tenant[s] >= 0 && c->block_slot[c->slot_tenant[s]] == s) c->block_slot[c->slot_tenant[s]] = -1;
    c->slot_tenant[s] = block;
    c->block_slot[block] = s;
    c->slot_state[s] = SLOT_FILLED;
    if (c->pause_resume) {
        if (!c->worker.joinable()) c->worker = std::thread(worker_main, c);
        {
            std::lock_guard<std::mutex> lk(c->mu);
            c->enq_count[s] = c->P(block).n_res_chunks;
            c->jobs.push_back(PrefetchJob{block, s, (hipStream_t)copy_stream});
        }
        c->cv.notify_all();
        return CF_OK;
    }
    return enqueue_block_copies(c, block, s, (hipStream_t)copy_stream, false);
}

int chunked_prefetch_wait(cf_ctx* c, int32_t block, int32_t chunk, void* compute_stream) {
    CF_TRY(check_block(c, block));
    const Plan& p = c->P(block);
    if (chunk < -1 || chunk >= p.n_chunks) return cf_fail(c, CF_ERR_ARG, "chunk %d out of range", chunk);
    const int last = chunk < 0 ? p.n_chunks - 1 : chunk;
    if (last < p.n_res_chunks) return CF_OK;
    // the copy stream is in order: waiting for `last` covers every earlier chunk
    return wait_chunk(c, block, last, (hipStream_t)compute_stream);
}

int dit_block_fwd(cf_ctx* c, int32_t block, const cf_block_io* io, void* compute_stream) {
    CF_TRY(check_block(c, block));
    if (!io) return cf_fail(c, CF_ERR_ARG, "null io");
    if (!io->x || !io->temb || !io->y) return cf_fail(c, CF_ERR_ARG, "x, temb and y are required");
    if (!io->workspace || io->workspace_bytes < c->ws_bytes || ((uintptr_t)io->workspace % 256))
        return cf_fail(c, CF_ERR_ARG, "workspace must be 256-byte aligned and at least %llu bytes", (unsigned long long)c->ws_bytes);
    if (((uintptr_t)io->x | (uintptr_t)io->y | (uintptr_t)io->temb) % 16) return cf_fail(c, CF_ERR_ARG, "x, y, temb must be 16-byte aligned");
    if ((io->rope_cos == nullptr) != (io->rope_sin == nullptr)) return cf_fail(c, CF_ERR_ARG, "rope_cos and rope_sin go together");
    if (((uintptr_t)io->rope_cos | (uintptr_t)io->rope_sin) % 16) return cf_fail(c, CF_ERR_ARG, "rope tables must be 16-byte aligned");
    const Plan& p = c->P(block);
    if (p.kind == CF_DOUBLE_STREAM && (!io->x_txt || !io->y_txt)) return cf_fail(c, CF_ERR_ARG, "double-stream needs x_txt and y_txt");
    if (p.kind == CF_DIT_CROSS && !io->ctx) return cf_fail(c, CF_ERR_ARG, "DiT block needs ctx");
    {
        // sample strides of the residual streams: 0 = dense, else at least one sample, 16-byte granular
        const int64_t nl = c->d.n_total / c->d.sp_degree, tl = c->d.n_txt_total / c->d.sp_degree;
        const int64_t x_rows = p.kind == CF_DOUBLE_STREAM ? nl - tl : nl;
        if (io->x_sample_stride && (io->x_sample_stride < x_rows * c->d.d || io->x_sample_stride % 4))
            return cf_fail(c, CF_ERR_ARG, "x_sample_stride must be 0 or a multiple of 4 that covers one sample's rows");
        if (io->x_txt_sample_stride && (io->x_txt_sample_stride < tl * c->d.d || io->x_txt_sample_stride % 4))
            return cf_fail(c, CF_ERR_ARG, "x_txt_sample_stride must be 0 or a multiple of 4 that covers one sample's rows");
    }
    if (!c->host[block]) return cf_fail(c, CF_ERR_STATE, "block %d has no registered host blob", block);
    CF_TRY(ensure_device(c));
    const int s = c->block_slot[block];
    const bool streamed = p.n_res_chunks < p.n_chunks;
    if (streamed && (s < 0 || c->slot_tenant[s] != block || c->slot_state[s] != SLOT_FILLED))
        return cf_fail(c, CF_ERR_STATE, "block %d: chunked_prefetch_begin must precede dit_block_fwd", block);

    // While collectives are emulated the host stays at most one block ahead of the GPU, streamed weights or not
    // (chunked_prefetch_begin bounds it the same way when chunks stream): waits between the compute and the
    // collective stream that are enqueued long before their events fire cost far more than waits that find
    // the event fired (measured: a fully resident step with collectives 18-22 ms unbounded, 14 ms bounded).
    if (c->comm_stream && c->comm_bytes && c->fwd_count >= 2)
        CF_HIP(c, hipEventSynchronize(c->fwd_ev[(c->fwd_count - 2) % 4]));

    Fwd F{c, block, (hipStream_t)compute_stream, view_of(c, block), io, carve(c->d, p.kind, (char*)io->workspace)};
    c->waited_upto = p.n_res_chunks - 1;
    if (streamed && c->adaptive_waits && !c->pause_resume && c->hidden_kind[p.kind]) {
        // blocks of this kind have been finding their weights in place: wait once, for the last chunk, and
        // launch every layer whole (Sec. 2.2's plain wait-then-forward)
        CF_TRY(wait_chunk(c, block, p.n_chunks - 1, (hipStream_t)compute_stream));
        c->waited_upto = p.n_chunks - 1;
        c->stats.blocks_one_wait++;
    }
    int rc;
    switch (p.kind) {
        case CF_SINGLE_STREAM: rc = fwd_single(F); break;
        case CF_DIT_CROSS: rc = fwd_dit(F); break;
        default: rc = fwd_double(F); break;
    }
    if (streamed) {
        // The slot's release must follow every chunk: a tail chunk that fed no layer is waited for here
        // (nothing to do when the layers' own waits reached the last chunk -- a wait on an event that fired
        // long ago still costs the stream tens of microseconds).  A forward that failed half way releases
        // its slot all the same, behind whatever it had enqueued, so that the next prefetch is not refused;
        // the caller gets the forward's error, the message of a failing release is dropped.
        const std::string fwd_err = c->err;
        int rel = CF_OK;
        if (c->waited_upto < p.n_chunks - 1) rel = chunked_prefetch_wait(c, block, -1, compute_stream);
        if (rel == CF_OK && hipEventRecord(c->done_ev[s], (hipStream_t)compute_stream) != hipSuccess)
            rel = cf_fail(c, CF_ERR_HIP, "recording the slot's release failed");
        c->slot_fwd_seq[s] = ++c->fwd_seq;
        c->done_valid[s] = rel == CF_OK;
        c->slot_state[s] = SLOT_CONSUMED;
        if (rc != CF_OK) c->err = fwd_err; else rc = rel;
    }
    if (rc != CF_OK) return rc;
    CF_HIP(c, hipEventRecord(c->fwd_ev[c->fwd_count % 4], (hipStream_t)compute_stream));
    c->fwd_count++;
    return CF_OK;
}

int cf_set_contention(cf_ctx* c, void* comm_stream, void* host_pinned, uint64_t host_bytes,
                      uint64_t bytes_per_collective, int32_t pause_resume) {
    if (!c) return CF_ERR_ARG;
    CF_TRY(ensure_device(c));
    worker_drain(c);
    CF_HIP(c, hipDeviceSynchronize());
    {
        // nothing is in flight any more: collectives of the previous setting are history
        std::lock_guard<std::mutex> lk(c->mu);
        for (auto& pc : c->comm_pending) { c->comm_ev_pool.push_back(pc.ready); c->comm_ev_pool.push_back(pc.done); }
        c->comm_pending.clear();
        c->cur_ready = c->cur_done = nullptr;
    }
    if (pause_resume < 0 || pause_resume > 2) return cf_fail(c, CF_ERR_ARG, "pause_resume must be 0, 1 or 2");
    if (!comm_stream) {
        c->comm_stream = nullptr;
        c->comm_bytes = 0;
        c->pause_resume = false;
        worker_stop(c);
        return CF_OK;
    }
    if (bytes_per_collective % 512) return cf_fail(c, CF_ERR_ARG, "bytes_per_collective must be a multiple of 512");
    if (bytes_per_collective) {
        if (!host_pinned || host_bytes < bytes_per_collective) return cf_fail(c, CF_ERR_ARG, "pinned host buffer too small");
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, host_pinned) != hipSuccess || attr.type != hipMemoryTypeHost) {
            (void)hipGetLastError();
            return cf_fail(c, CF_ERR_ARG, "collective host buffer must be pinned host memory");
        }
        if (c->comm_dev) (void)hipFree(c->comm_dev);
        c->comm_dev = nullptr;
        if (hipMalloc((void**)&c->comm_dev, bytes_per_collective) != hipSuccess) {
            (void)hipGetLastError();
            return cf_fail(c, CF_ERR_NOMEM, "hipMalloc of the collective buffer failed");
        }
    }
    c->comm_stream = (hipStream_t)comm_stream;
    c->comm_host = (uint8_t*)host_pinned;
    c->comm_bytes = bytes_per_collective;
    c->pause_resume = pause_resume != 0;
    c->pause_depth = pause_resume == 2 ? 2 : 1;
    if (!c->pause_resume) worker_stop(c);
    return CF_OK;
}

int cf_comm_begin(cf_ctx* c, void* comm_stream, void* compute_stream) {
    if (!c || !comm_stream) return CF_ERR_ARG;
    CF_TRY(ensure_device(c));
    return cf_comm_begin_impl(c, (hipStream_t)comm_stream, (hipStream_t)compute_stream);
}

int cf_comm_end(cf_ctx* c, void* comm_stream, void* compute_stream) {
    if (!c || !comm_stream) return CF_ERR_ARG;
    CF_TRY(ensure_device(c));
    return cf_comm_end_impl(c, (hipStream_t)comm_stream, (hipStream_t)compute_stream);
}

int cf_checksum_block(cf_ctx* c, int32_t block, uint64_t* host_out, void* stream) {
    CF_TRY(check_block(c, block));
    if (!host_out) return cf_fail(c, CF_ERR_ARG, "null output");
    CF_TRY(ensure_device(c));
    hipStream_t s = (hipStream_t)stream;
    const Plan& p = c->P(block);
    if (p.n_res_chunks < p.n_chunks) CF_TRY(chunked_prefetch_wait(c, block, -1, stream));
    if (!c->checksum_dev && hipMalloc((void**)&c->checksum_dev, 8ull * c->max_chunks) != hipSuccess) {
        (void)hipGetLastError();
        c->checksum_dev = nullptr;
        return cf_fail(c, CF_ERR_NOMEM, "hipMalloc of the checksum words failed");
    }
    uint64_t* const dev = c->checksum_dev;
    const WView v = view_of(c, block);
    int rc = CF_OK;
    for (int k = 0; k < p.n_chunks && rc == CF_OK; ++k) {
        const uint64_t b = chunk_begin(c, k), e = chunk_end(c, p, k);
        const char* src = (b < v.split ? v.lo : v.hi) + b;
        hipError_t he = checksum_launch(src, e - b, b / 8, dev + k, s);
        if (he != hipSuccess) rc = cf_fail(c, CF_ERR_HIP, "checksum launch failed: %s", hipGetErrorString(he));
    }
    if (rc == CF_OK && hipMemcpyAsync(host_out, dev, 8ull * p.n_chunks, hipMemcpyDeviceToHost, s) != hipSuccess) rc = cf_fail(c, CF_ERR_HIP, "checksum copy failed");
    if (hipStreamSynchronize(s) != hipSuccess && rc == CF_OK) rc = cf_fail(c, CF_ERR_HIP, "checksum sync failed");
    return rc;
}

int cf_read_block(cf_ctx* c, int32_t block, void* host_out, void* stream) {
    CF_TRY(check_block(c, block));
    if (!host_out) return cf_fail(c, CF_ERR_ARG, "null output");
    CF_TRY(ensure_device(c));
    hipStream_t s = (hipStream_t)stream;
    const Plan& p = c->P(block);
    if (p.n_res_chunks < p.n_chunks) CF_TRY(chunked_prefetch_wait(c, block, -1, stream));
    if (p.res_bytes) {
        if (!c->res_buf[block]) return cf_fail(c, CF_ERR_STATE, "block %d not registered", block);
        CF_HIP(c, hipMemcpyAsync(host_out, c->res_buf[block], p.res_bytes, hipMemcpyDeviceToHost, s));
    }
    if (p.res_bytes < p.blob_bytes)
        CF_HIP(c, hipMemcpyAsync((char*)host_out + p.res_bytes, c->slot[c->block_slot[block]], p.blob_bytes - p.res_bytes, hipMemcpyDeviceToHost, s));
    CF_HIP(c, hipStreamSynchronize(s));
    return CF_OK;
}

int cf_stats(cf_ctx* c, cf_stats_t* out) {
    if (!c || !out) return CF_ERR_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    *out = c->stats;
    // resident and blob bytes per block, averaged over the model's blocks; weight memory (Sec. 3.3)
    // = every block's resident part + two staging slots sized for the largest streamed part
    uint64_t res = 0, all = 0, slot = 0;
    for (int k : c->block_kind) { res += c->plan[k].res_bytes; all += c->plan[k].blob_bytes; }
    for (int k = 0; k < 3; ++k)
        if (c->plan[k].kind >= 0) slot = std::max(slot, c->plan[k].blob_bytes - c->plan[k].res_bytes);
    out->resident_bytes = res / c->d.n_blocks;
    out->blob_bytes = all / c->d.n_blocks;
    out->weight_memory_bytes = res + 2 * slot;
    out->model_resident_bytes = res;
    out->model_blob_bytes = all;
    return CF_OK;
}

int cf_stats_reset(cf_ctx* c) {
    if (!c) return CF_ERR_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    c->stats = cf_stats_t{};
    return CF_OK;
}

int cf_set_adaptive_waits(cf_ctx* c, int32_t on) {
    if (!c) return CF_ERR_ARG;
    c->adaptive_waits = on != 0;
    for (bool& h : c->hidden_kind) h = false;
    return CF_OK;
}

int cf_set_profiling(cf_ctx* c, int32_t on) {
    if (!c) return CF_ERR_ARG;
    c->profiling = on != 0;
    return CF_OK;
}

int cf_kernel_times(cf_ctx* c, cf_kernel_time* out, int32_t* n) {
    if (!c || !n) return CF_ERR_ARG;
    worker_drain(c);
    CF_TRY(prof_resolve(c));
    int cnt = 0;
    for (auto& k : c->ktimes)
        if (k.launches) ++cnt;
    if (out) {
        if (*n < cnt) return cf_fail(c, CF_ERR_ARG, "need room for %d kernel records", cnt);
        int i = 0;
        for (auto& k : c->ktimes)
            if (k.launches) out[i++] = k;
    }
    *n = cnt;
    return CF_OK;
}

int cf_kernel_times_reset(cf_ctx* c) {
    if (!c) return CF_ERR_ARG;
    CF_TRY(prof_resolve(c));
    c->ktimes.clear();
    return CF_OK;
}

int cf_sync(cf_ctx* c) {
    if (!c) return CF_ERR_ARG;
    worker_drain(c);
    CF_HIP(c, hipDeviceSynchronize());
    if (!c->worker_err.empty()) return cf_fail(c, CF_ERR_HIP, "prefetch worker: %s", c->worker_err.c_str());
    return CF_OK;
}

// ---- single kernels -----------------------------------------------------------------------
static WView flat_view(const void* blob) { return WView{(const char*)blob, (const char*)blob, ~0ull}; }

int cf_op_linear(const uint16_t* A, int32_t lda, const void* blob, uint64_t w_off, int64_t bias_off, int32_t M, int32_t N,
                 int32_t K, int32_t n0, int32_t n1, int32_t n_split, uint16_t* out0, int32_t ld0, uint16_t* out1,
                 int32_t ld1, int32_t gelu_erf, void* stream) {
    if (!A || !blob) return cf_fail(nullptr, CF_ERR_ARG, "null operand");
    GemmArgs g{};
    g.A = (const bf16*)A; g.lda = lda; g.W = flat_view(blob); g.w_off = w_off;
    g.has_bias = bias_off >= 0; g.bias_off = bias_off >= 0 ? (uint64_t)bias_off : 0;
    g.M = M; g.N = N; g.K = K; g.n0 = n0; g.n1 = n1; g.epi = EPI_SPLIT_GELU;
    g.out0 = (bf16*)out0; g.ld0 = ld0; g.n_split = n_split; g.out1 = (bf16*)out1; g.ld1 = ld1; g.col1_off = 0;
    g.act_erf = gelu_erf != 0;
    if (const char* msg = gemm_check(g)) return cf_fail(nullptr, CF_ERR_ARG, "%s", msg);
    hipError_t e = gemm_launch(g, (hipStream_t)stream);
    return e == hipSuccess ? CF_OK : cf_fail(nullptr, CF_ERR_HIP, "gemm launch: %s", hipGetErrorString(e));
}

int cf_op_linear_residual(const uint16_t* A, int32_t lda, const void* blob, uint64_t w_off, int64_t bias_off, int32_t M,
                          int32_t N, int32_t K, const float* resid, const float* gate, float* y, void* stream) {
    if (!A || !blob) return cf_fail(nullptr, CF_ERR_ARG, "null operand");
    GemmArgs g{};
    g.A = (const bf16*)A; g.lda = lda; g.W = flat_view(blob); g.w_off = w_off;
    g.has_bias = bias_off >= 0; g.bias_off = bias_off >= 0 ? (uint64_t)bias_off : 0;
    g.M = M; g.N = N; g.K = K; g.n0 = 0; g.n1 = N; g.epi = EPI_GATE_RESID;
    g.resid = resid; g.gate = gate; g.y = y; g.ldy = N;
    if (const char* msg = gemm_check(g)) return cf_fail(nullptr, CF_ERR_ARG, "%s", msg);
    hipError_t e = gemm_launch(g, (hipStream_t)stream);
    return e == hipSuccess ? CF_OK : cf_fail(nullptr, CF_ERR_HIP, "gemm launch: %s", hipGetErrorString(e));
}

int cf_op_attention(const uint16_t* Q, const uint16_t* K, const uint16_t* Vt, uint16_t* O, int32_t H, int32_t nq,
                    int32_t nk, int32_t nk_pad, int32_t hd, void* stream) {
    AttnArgs a{};
    a.Q = (const bf16*)Q; a.K = (const bf16*)K; a.Vt = (const bf16*)Vt; a.O = (bf16*)O;
    a.o_hs = (long)nq * hd; a.o_qs = hd; a.H = H; a.nq = nq; a.nk = nk; a.nk_pad = nk_pad; a.hd = hd;
    a.scale = 1.0f / sqrtf((float)hd);
    if (const char* msg = attn_check(a)) return cf_fail(nullptr, CF_ERR_ARG, "%s", msg);
    hipError_t e = attn_launch(a, (hipStream_t)stream);
    return e == hipSuccess ? CF_OK : cf_fail(nullptr, CF_ERR_HIP, "attention launch: %s", hipGetErrorString(e));
}

int cf_op_ln_modulate(const float* x, const float* shift, const float* scale, uint16_t* xn, int32_t rows, int32_t d,
                      void* stream) {
    if (!x || !shift || !scale || !xn) return cf_fail(nullptr, CF_ERR_ARG, "null operand");
    hipError_t e = ln_modulate_launch(x, shift, scale, (bf16*)xn, rows, d, d, 0, 0, 0, (hipStream_t)stream);
    return e == hipSuccess ? CF_OK : cf_fail(nullptr, CF_ERR_ARG, "ln_modulate: %s", hipGetErrorString(e));
}

int cf_op_modvec(const void* blob, uint64_t w_off, uint64_t b_off, const float* t, float* m, int32_t n, int32_t K,
                 void* stream) {
    if (!blob || !t || !m || (w_off % 16) || (K % 8)) return cf_fail(nullptr, CF_ERR_ARG, "bad modvec operands");
    hipError_t e = modvec_launch(flat_view(blob), w_off, b_off, t, m, 0, n, K, 1, 0, (hipStream_t)stream);
    return e == hipSuccess ? CF_OK : cf_fail(nullptr, CF_ERR_HIP, "modvec: %s", hipGetErrorString(e));
}

int cf_op_mfma_rate(int32_t iters, int32_t random_operands, float* out, void* stream) {
    if (iters <= 0 || iters > (1 << 24) || !out) return cf_fail(nullptr, CF_ERR_ARG, "mfma_rate: bad arguments");
    hipError_t e = mfma_rate_launch(iters, random_operands != 0, out, (hipStream_t)stream);
    return e == hipSuccess ? CF_OK : cf_fail(nullptr, CF_ERR_HIP, "mfma_rate: %s", hipGetErrorString(e));
}

int cf_op_mix_rate(int32_t iters, int32_t waves, int32_t reads_per_16, int32_t valu_per_mfma, int32_t exp_per_mfma, float* out,
                   void* stream) {
    if (iters <= 0 || iters > (1 << 24) || !out) return cf_fail(nullptr, CF_ERR_ARG, "mix_rate: bad arguments");
    hipError_t e = mix_rate_launch(iters, waves, reads_per_16, valu_per_mfma, exp_per_mfma, out, (hipStream_t)stream);
    if (e == hipErrorInvalidValue) { (void)hipGetLastError(); return cf_fail(nullptr, CF_ERR_ARG, "mix_rate: this instruction mix is not built"); }
    return e == hipSuccess ? CF_OK : cf_fail(nullptr, CF_ERR_HIP, "mix_rate: %s", hipGetErrorString(e));
}

int cf_op_checksum(const void* data, uint64_t bytes, uint64_t first_word, uint64_t* host_out, void* stream) {
    if (!data || !host_out) return cf_fail(nullptr, CF_ERR_ARG, "null operand");
    uint64_t* dev = nullptr;
    if (hipMalloc((void**)&dev, 8) != hipSuccess) { (void)hipGetLastError(); return cf_fail(nullptr, CF_ERR_NOMEM, "hipMalloc failed"); }
    hipError_t e = checksum_launch(data, bytes, first_word, dev, (hipStream_t)stream);
    if (e == hipSuccess) e = hipMemcpyAsync(host_out, dev, 8, hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    (void)hipFree(dev);
    return e == hipSuccess ? CF_OK : cf_fail(nullptr, CF_ERR_HIP, "checksum: %s", hipGetErrorString(e));
}

}  // extern "C"

namespace {

int cf_comm_begin_impl(cf_ctx* c, hipStream_t comm, hipStream_t compute) {
    if (c->pause_resume) {
        // pause/resume: this collective gets an event pair of its own, which the prefetch worker polls --
        // `ready` tells it, in GPU time, that the compute stream has reached the collective (Sec. 3.2: the
        // flag goes up when the collective is issued), `done` is what it parks the copy stream on
        std::lock_guard<std::mutex> lk(c->mu);
        retire_finished_collectives(c);                // also when no chunk streams and the worker never looks
        for (hipEvent_t* e : {&c->cur_ready, &c->cur_done}) {
            if (!c->comm_ev_pool.empty()) { *e = c->comm_ev_pool.back(); c->comm_ev_pool.pop_back(); }
            else CF_HIP(c, hipEventCreateWithFlags(e, hipEventDisableTiming));
        }
        CF_HIP(c, hipEventRecord(c->cur_ready, compute));
        c->comm_pending.push_back(PendingComm{c->cur_ready, c->cur_done, false, false});
    } else {
        c->cur_ready = c->comm_ready_ev;
        c->cur_done = c->comm_done_ev;
        CF_HIP(c, hipEventRecord(c->cur_ready, compute));
    }
    // the collective may start once the compute stream has produced its operands
    CF_HIP(c, hipStreamWaitEvent(comm, c->cur_ready, 0));
    return CF_OK;
}

int cf_comm_end_impl(cf_ctx* c, hipStream_t comm, hipStream_t compute) {
    if (!c->cur_done) return cf_fail(c, CF_ERR_STATE, "cf_comm_end without cf_comm_begin");
    {
        std::lock_guard<std::mutex> lk(c->mu);
        CF_HIP(c, hipEventRecord(c->cur_done, comm));
        if (c->pause_resume && !c->comm_pending.empty() && c->comm_pending.back().done == c->cur_done)
            c->comm_pending.back().done_recorded = true;
    }
    c->cv.notify_all();
    ProfScope ps(c, compute, K_COMM_WAIT, 0, 0);
    CF_HIP(c, hipStreamWaitEvent(compute, c->cur_done, 0));
    return CF_OK;
}

TokenMap identity_map(int rows) { return TokenMap{rows, rows, 0, rows, rows, 0}; }

GemmArgs plain_linear(const bf16* A, int lda, int M, bf16* out, int ld) {
    GemmArgs g{};
    g.A = A; g.lda = lda; g.M = M; g.epi = EPI_SPLIT_GELU;
    g.out0 = out; g.ld0 = ld; g.n_split = 1 << 30;      // clamped to N below: no GELU half
    return g;
}
GemmArgs gelu_linear(const bf16* A, int lda, int M, bf16* out, int ld) {
    GemmArgs g{};
    g.A = A; g.lda = lda; g.M = M; g.epi = EPI_SPLIT_GELU;
    g.n_split = 0; g.out1 = out; g.ld1 = ld; g.col1_off = 0;
    return g;
}
GemmArgs resid_linear(const bf16* A, int lda, int M, const float* resid, const float* gate, float* y, int ld) {
    GemmArgs g{};
    g.A = A; g.lda = lda; g.M = M; g.epi = EPI_GATE_RESID;
    g.resid = resid; g.gate = gate; g.y = y; g.ldy = ld;
    return g;
}

// ---- DiT block (App. B): modulated self-attention, cross-attention to the text context
// (affine pre-norm, no gate, text K/V computed by every rank), modulated FFN
int fwd_dit(Fwd& F) {
    cf_ctx* c = F.c;
    const cf_model_desc& m = c->d;
    const int d = m.d, f = m.f, nl = m.n_total / m.sp_degree, H = m.n_heads, hd = m.head_dim, lc = m.l_ctx;
    const int B = batch_of(m), rows = B * nl, rps = B > 1 ? nl : 0;
    const cf_block_io* io = F.io;
    Ws& w = F.ws;
    const long mod_bs = 6L * d, xs = x_stride(io, (long)nl * d), dense = (long)nl * d;
    CF_TRY(run_modvec(F, "w_mod", "b_mod", io->temb, w.mod, mod_bs));
    const float *sh1 = w.mod, *sc1 = w.mod + d, *g1 = w.mod + 2 * d, *sh2 = w.mod + 3 * d, *sc2 = w.mod + 4 * d,
                *g2 = w.mod + 5 * d;
    // self-attention
    CF_TRY(run_ln_mod(F, io->x, sh1, sc1, w.xn, rows, rps, xs, mod_bs));
    if (m.qk_rmsnorm) { CF_TRY(need(F, T(F, "q_norm"))); CF_TRY(need(F, T(F, "k_norm"))); }
    CF_TRY(run_linear(F, K_QKV, "w_qkv", "b_qkv", plain_linear(w.xn, d, rows, w.qkv, 3 * d)));
    RelayoutArgs r = relayout_for(F, w.qkv, nl, 0, "q_norm", "k_norm");
    CF_TRY(run_joint_attention(F, &r, 1, AttnOut{w.c, nullptr, d, dense, 0}));
    CF_TRY(run_linear(F, K_OUT, "w_o", "b_o", batched(resid_linear(w.c, d, rows, io->x, g1, w.x1, d), B, nl, mod_bs, xs, dense)));
    // cross-attention: queries from the local tokens (all heads), keys/values from the context
    CF_TRY(need(F, T(F, "ln_c_w")));
    CF_TRY(need(F, T(F, "ln_c_b")));
    {
        ProfScope ps(c, F.s, K_LN, 0, 6.0 * rows * d);
        CF_HIP(c, ln_affine_launch(w.x1, F.W, T(F, "ln_c_w").off, T(F, "ln_c_b").off, w.xn, rows, d, F.s));
    }
    if (m.qk_rmsnorm) { CF_TRY(need(F, T(F, "cq_norm"))); CF_TRY(need(F, T(F, "ck_norm"))); }
    {
        // the query projection of the local tokens and the K/V projection of the context are independent
        const std::string wn[2] = {"w_cq", "w_ckv"}, bn[2] = {"b_cq", "b_ckv"};
        const GemmArgs g[2] = {plain_linear(w.xn, d, rows, w.qkv, d), plain_linear((const bf16*)io->ctx, d, B * lc, w.ckv, 2 * d)};
        CF_TRY(run_linear_pair(F, K_CROSS_Q, wn, bn, g));
    }
    const int lpad = n_pad_of(lc);
    for (int b = 0; b < B; ++b) {
        RelayoutArgs rq{};
        rq.src = w.qkv + (size_t)b * nl * d; rq.ld = d; rq.rows = nl; rq.col_q = 0; rq.col_k = -1; rq.col_v = -1;
        rq.n_heads = H; rq.h0 = 0; rq.h_local = H; rq.hd = hd; rq.W = F.W; rq.has_norm = m.qk_rmsnorm;
        if (m.qk_rmsnorm) { rq.qn_off = T(F, "cq_norm").off; rq.kn_off = T(F, "ck_norm").off; }
        rq.map = identity_map(nl); rq.row0 = 0; rq.Q = w.cQ + (size_t)b * nl * d; rq.K = nullptr; rq.Vt = nullptr; rq.n_pad = 0;
        RelayoutArgs rk = rq;
        rk.src = w.ckv + (size_t)b * lc * 2 * d; rk.ld = 2 * d; rk.rows = lc; rk.col_q = -1; rk.col_k = 0; rk.col_v = d;
        rk.map = identity_map(lc); rk.Q = nullptr; rk.K = w.cK + (size_t)b * lc * d; rk.Vt = w.cVt + (size_t)b * d * lpad;
        rk.n_pad = lpad;
        ProfScope ps(c, F.s, K_RELAYOUT, 0, 2.0 * 2 * ((double)nl * d + 2.0 * lc * d));
        CF_HIP(c, relayout_launch(rq, F.s));
        CF_HIP(c, relayout_launch(rk, F.s));
    }
    {
        AttnArgs a{};
        a.Q = w.cQ; a.K = w.cK; a.Vt = w.cVt; a.O = w.c; a.o_hs = hd; a.o_qs = d; a.o_bs = dense;
        a.H = B * H; a.hps = H; a.nq = nl; a.nk = lc; a.nk_pad = lpad; a.hd = hd; a.scale = 1.0f / sqrtf((float)hd);
        if (const char* msg = attn_check(a)) return cf_fail(c, CF_ERR_ARG, "%s", msg);
        ProfScope ps(c, F.s, K_CROSS_ATTN, 4.0 * B * H * (double)nl * lc * hd, 0);
        CF_HIP(c, attn_launch(a, F.s));
    }
    CF_TRY(run_linear(F, K_CROSS_OUT, "w_co", "b_co", resid_linear(w.c, d, rows, w.x1, nullptr, w.x2, d)));
    // FFN
    CF_TRY(run_ln_mod(F, w.x2, sh2, sc2, w.xn, rows, rps, dense, mod_bs));
    CF_TRY(run_linear(F, K_UP, "w_up", "b_up", gelu_linear(w.xn, d, rows, w.up, f)));
    return run_linear(F, K_DOWN, "w_down", "b_down", batched(resid_linear(w.up, f, rows, w.x2, g2, io->y, d), B, nl, mod_bs, dense, xs));
}

// ---- MM-DiT double-stream block (App. B): per-stream weights, joint attention over the
// concatenation (text rows, then image rows).  Local rows: this rank's text rows, then image rows.
int fwd_double(Fwd& F) {
    cf_ctx* c = F.c;
    const cf_model_desc& m = c->d;
    const int d = m.d, f = m.f, nl = m.n_total / m.sp_degree, tl = m.n_txt_total / m.sp_degree, B = batch_of(m);
    const cf_block_io* io = F.io;
    Ws& w = F.ws;
    static const char* st[2] = {"txt", "img"};
    auto nm = [](const char* s, const char* t) { return std::string(s) + "_" + t; };
    // workspace rows: all samples' text rows, then all samples' image rows
    const int per[2] = {tl, nl - tl};                       // rows of one sample
    const int row0[2] = {0, B * tl}, rows[2] = {B * tl, B * (nl - tl)};
    const int rps[2] = {B > 1 ? per[0] : 0, B > 1 ? per[1] : 0};
    const float* xin[2] = {io->x_txt, io->x};
    float* yout[2] = {io->y_txt, io->y};
    const long xs[2] = {x_txt_stride(io, (long)per[0] * d), x_stride(io, (long)per[1] * d)};
    const long dense[2] = {(long)per[0] * d, (long)per[1] * d};
    const long mod_bs = 12L * d;
    for (int s = 0; s < 2; ++s) CF_TRY(run_modvec(F, nm(st[s], "w_mod"), nm(st[s], "b_mod"), io->temb, w.mod + 6 * d * s, mod_bs));
    auto mod = [&](int s, int i) { return w.mod + 6 * d * s + i * d; };
    for (int s = 0; s < 2; ++s)
        CF_TRY(run_ln_mod(F, xin[s], mod(s, 0), mod(s, 1), w.xn + (size_t)row0[s] * d, rows[s], rps[s], xs[s], mod_bs));
    RelayoutArgs parts[2];
    auto names = [&](const char* t, std::string (&out)[2]) { out[0] = nm(st[0], t); out[1] = nm(st[1], t); };
    std::string wn[2], bn[2];
    {
        const GemmArgs g[2] = {plain_linear(w.xn + (size_t)row0[0] * d, d, rows[0], w.qkv + (size_t)row0[0] * 3 * d, 3 * d),
                               plain_linear(w.xn + (size_t)row0[1] * d, d, rows[1], w.qkv + (size_t)row0[1] * 3 * d, 3 * d)};
        names("w_qkv", wn); names("b_qkv", bn);
        CF_TRY(run_linear_pair(F, K_QKV, wn, bn, g));
    }
    for (int s = 0; s < 2; ++s) {
        if (m.qk_rmsnorm) { CF_TRY(need(F, T(F, nm(st[s], "q_norm")))); CF_TRY(need(F, T(F, nm(st[s], "k_norm")))); }
        parts[s] = relayout_for(F, w.qkv + (size_t)row0[s] * 3 * d, per[s], s ? tl : 0, nm(st[s], "q_norm"), nm(st[s], "k_norm"));
    }
    // one sample: its image rows follow its text rows in w.c; a batch: the streams' regions are apart
    CF_TRY(run_joint_attention(F, parts, 2, B > 1 ? AttnOut{w.c, w.c + (size_t)row0[1] * d, d, dense[0], dense[1]}
                                                  : AttnOut{w.c, nullptr, d, (long)nl * d, 0}));
    {
        GemmArgs g[2];
        for (int s = 0; s < 2; ++s)
            g[s] = batched(resid_linear(w.c + (size_t)row0[s] * d, d, rows[s], xin[s], mod(s, 2), w.x1 + (size_t)row0[s] * d, d),
                           B, per[s], mod_bs, xs[s], dense[s]);
        names("w_o", wn); names("b_o", bn);
        CF_TRY(run_linear_pair(F, K_OUT, wn, bn, g));
    }
    for (int s = 0; s < 2; ++s)
        CF_TRY(run_ln_mod(F, w.x1 + (size_t)row0[s] * d, mod(s, 3), mod(s, 4), w.xn + (size_t)row0[s] * d, rows[s], rps[s], dense[s], mod_bs));
    {
        GemmArgs g[2];
        for (int s = 0; s < 2; ++s) g[s] = gelu_linear(w.xn + (size_t)row0[s] * d, d, rows[s], w.up + (size_t)row0[s] * f, f);
        names("w_up", wn); names("b_up", bn);
        CF_TRY(run_linear_pair(F, K_UP, wn, bn, g));
    }
    {
        GemmArgs g[2];
        for (int s = 0; s < 2; ++s)
            g[s] = batched(resid_linear(w.up + (size_t)row0[s] * f, f, rows[s], w.x1 + (size_t)row0[s] * d, mod(s, 5), yout[s], d),
                           B, per[s], mod_bs, dense[s], xs[s]);
        names("w_down", wn); names("b_down", bn);
        CF_TRY(run_linear_pair(F, K_DOWN, wn, bn, g));
    }
    return CF_OK;
}

}  // namespace

const TensorDesc* cf_find(const Plan& c, const char* name) {
    for (auto& t : c.tensors)
        if (t.name == name) return &t;
    return nullptr;
}
