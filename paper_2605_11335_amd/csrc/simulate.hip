// Chunk-level model of one denoising step under layerwise offloading, and the memory-latency
// dial built on it.  Host arithmetic only.
//
// Sec. 3.1 states the first-order condition (a block's prefetch is hidden iff T_comp >= T_pref);
// Sec. 3.2 cuts the prefetch into chunks and Sec. 3.3 keeps a prefix of them resident.  This
// model follows the two streams the scheduler actually drives, chunk by chunk:
//   copy stream     the streamed chunks of block i+1 go out in order, back to back, once the
//                   chunks of block i are out and block i-1 (last tenant of the slot) is done;
//   compute stream  a block's compute is split into one segment per chunk -- the work that the
//                   bytes of that chunk make possible -- and segment k starts when segment k-1
//                   has ended and chunk k has landed (resident chunks never wait).
// A segment's share of the block's compute time is the share of the block's matrix FLOPs that the
// chunk completes: a linear layer is taken in row groups of about one round of tiles (row_group),
// each booked on the chunk that holds its last byte; attention is attributed to the chunk that completes the QKV
// projection (cross-attention: the context K/V projection).  With one chunk per block and
// nothing resident the step time is the sum over blocks of max(T_comp, T_pref).
#include <algorithm>
#include <cmath>
#include <cstring>

#include "context.h"

namespace {

// activation rows a weight matrix multiplies, by tensor name
double rows_of(const cf_model_desc& m, int kind, const std::string& name) {
    const double B = m.batch > 0 ? m.batch : 1;
    const double nl = B * m.n_total / m.sp_degree;
    if (kind == CF_DIT_CROSS) return name == "w_ckv" ? B * m.l_ctx : nl;
    if (kind == CF_DOUBLE_STREAM) {
        const double tl = B * m.n_txt_total / m.sp_degree;
        return name.rfind("txt_", 0) == 0 ? tl : nl - tl;
    }
    return nl;
}

// Rows of output features per row group of a linear layer on `m_rows` tokens: as many 256-wide
// feature tiles as give 256 tiles (one per CU) together with the 256-row token tiles.  The
// scheduler's panels are made of about such rounds.
int row_group(int m_rows) {
    const int tiles_m = std::max(1, (m_rows + 255) / 256);
    return 256 * ((256 + tiles_m - 1) / tiles_m);
}

// per-chunk share of one block's compute (sums to 1)
std::vector<double> segment_shares(const cf_model_desc& m, const Plan& p, uint64_t chunk_bytes) {
    std::vector<double> seg(p.n_chunks, 0.0);
    const double B = m.batch > 0 ? m.batch : 1;
    const double nl = (double)m.n_total / m.sp_degree, hl = (double)m.n_heads / m.sp_degree;
    const char* attn_after = p.kind == CF_SINGLE_STREAM ? "w1" : (p.kind == CF_DIT_CROSS ? "w_qkv" : "img_w_qkv");
    for (const TensorDesc& t : p.tensors) {
        if (t.rows <= 1) continue;                              // biases and norm weights: no matrix work
        const bool modvec = t.name.find("w_mod") != std::string::npos;
        const double act = modvec ? B : rows_of(m, p.kind, t.name);
        // a row group counts once its last byte has landed; the modulation matrix-vector product
        // goes 8 rows at a time
        const uint64_t G = modvec ? 8 : (uint64_t)row_group((int)act), row_bytes = 2ull * t.cols;
        for (uint64_t r0 = 0; r0 < t.rows; r0 += G) {
            const uint64_t r1 = std::min<uint64_t>(t.rows, r0 + G);
            seg[(t.off + r1 * row_bytes - 1) / chunk_bytes] += 2.0 * act * (double)(r1 - r0) * t.cols;
        }
        const uint64_t last = (t.off + t.bytes() - 1) / chunk_bytes;
        if (t.name == attn_after) seg[last] += 4.0 * B * hl * (double)m.n_total * m.n_total * m.head_dim;
        if (t.name == "w_ckv") seg[last] += 4.0 * B * m.n_heads * nl * m.l_ctx * m.head_dim;
    }
    double sum = 0;
    for (double v : seg) sum += v;
    for (double& v : seg) v /= sum;
    return seg;
}

struct SimPlan {
    Plan plan;
    std::vector<double> share;
    int n_res = 0;
    uint64_t res_bytes = 0;
};

int simulate(const cf_ctx* c, uint64_t chunk_bytes, double r, const cf_machine_t& mach, cf_sim_result* out) {
    const int L = c->d.n_blocks;
    SimPlan sp[3];
    uint64_t slot = 0, res_all = 0, blob_all = 0;
    double comp_all = 0;
    for (int k : c->block_kind) {
        SimPlan& s = sp[k];
        if (s.plan.kind < 0) {
            plan_layout(&s.plan, c->d, k, chunk_bytes);
            s.share = segment_shares(c->d, s.plan, chunk_bytes);
            s.n_res = (int)std::floor(r * s.plan.n_chunks + 0.5);
            s.res_bytes = s.n_res ? std::min(s.plan.blob_bytes, (uint64_t)s.n_res * chunk_bytes) : 0;
            slot = std::max(slot, s.plan.blob_bytes - s.res_bytes);
            if (!(mach.t_comp_ms[k] > 0)) return cf_fail(c, CF_ERR_ARG, "t_comp_ms[%d] must be positive", k);
        }
        res_all += s.res_bytes;
        blob_all += s.plan.blob_bytes;
        comp_all += mach.t_comp_ms[k];
    }
    const double ms_per_byte = 1e3 / (mach.link_gbs * 1e9), ovh = mach.chunk_overhead_us * 1e-3;
    // block instances i = step * L + l; done[i] = end of compute, copy_end = end of the copy stream's work
    const int steps = 4, n = steps * L;
    std::vector<double> done(n + 1, 0.0), begin_t(n + 1, 0.0);
    std::vector<std::vector<double>> arrive(n);
    double copy_end = 0;
    auto enqueue_copies = [&](int i, double issued) {
        const SimPlan& s = sp[c->block_kind[i % L]];
        double t = std::max(copy_end, issued);
        if (i >= 2) t = std::max(t, done[i - 2]);               // the slot's last tenant has been consumed
        arrive[i].assign(s.plan.n_chunks, 0.0);
        for (int k = s.n_res; k < s.plan.n_chunks; ++k) {
            const uint64_t b = (uint64_t)k * chunk_bytes, e = std::min(s.plan.blob_bytes, b + chunk_bytes);
            t += ovh + (double)(e - b) * ms_per_byte;
            arrive[i][k] = t;
        }
        copy_end = t;
    };
    enqueue_copies(0, 0.0);
    for (int i = 0; i < n; ++i) {
        const SimPlan& s = sp[c->block_kind[i % L]];
        double t = i ? done[i - 1] : 0.0;
        if (i + 1 < n) enqueue_copies(i + 1, t);               // prefetch of the next block is issued first (Sec. 2.2)
        for (int k = 0; k < s.plan.n_chunks; ++k) {
            if (k >= s.n_res) t = std::max(t, arrive[i][k]);
            t += s.share[k] * mach.t_comp_ms[s.plan.kind];
        }
        done[i] = t;
    }
    memset(out, 0, sizeof *out);
    out->step_ms = done[n - 1] - done[n - 1 - L];
    out->compute_ms = comp_all;
    out->exposed_ms = out->step_ms - comp_all;
    out->weight_memory_bytes = res_all + 2 * slot;
    out->h2d_bytes_per_step = blob_all - res_all;
    out->resident_fraction = (double)res_all / (double)blob_all;
    return CF_OK;
}

}  // namespace

extern "C" {

int cf_simulate(const cf_ctx* c, double r, const cf_machine_t* mach, cf_sim_result* out) {
    if (!c || !mach || !out) return CF_ERR_ARG;
    if (!(r >= 0.0 && r <= 1.0)) return cf_fail(c, CF_ERR_ARG, "resident fraction %g outside [0,1]", r);
    if (!(mach->link_gbs > 0) || mach->chunk_overhead_us < 0) return cf_fail(c, CF_ERR_ARG, "link_gbs must be positive, chunk_overhead_us non-negative");
    return simulate(c, c->chunk_bytes, r, *mach, out);
}

int cf_tune(const cf_ctx* c, const cf_machine_t* mach, const uint64_t* chunk_candidates, int32_t n_candidates,
            int32_t r_steps, uint64_t memory_budget_bytes, double step_target_ms, cf_tune_choice* out) {
    if (!c || !mach || !chunk_candidates || n_candidates <= 0 || r_steps <= 0 || !out) return CF_ERR_ARG;
    if (!(mach->link_gbs > 0) || mach->chunk_overhead_us < 0) return cf_fail(c, CF_ERR_ARG, "link_gbs must be positive, chunk_overhead_us non-negative");
    if ((memory_budget_bytes != 0) == (step_target_ms > 0))
        return cf_fail(c, CF_ERR_ARG, "give either a memory budget or a step-time target");
    bool have = false;
    cf_tune_choice best{};
    for (int ci = 0; ci < n_candidates; ++ci) {
        const uint64_t cb = chunk_candidates[ci];
        if (cb == 0 || cb % 256) return cf_fail(c, CF_ERR_ARG, "chunk candidate %d is not a positive multiple of 256", ci);
        for (int ri = 0; ri <= r_steps; ++ri) {
            cf_tune_choice t{};
            t.chunk_bytes = cb;
            t.r = (double)ri / r_steps;
            CF_TRY(simulate(c, cb, t.r, *mach, &t.sim));
            const bool ok = memory_budget_bytes ? t.sim.weight_memory_bytes <= memory_budget_bytes
                                                : t.sim.step_ms <= step_target_ms;
            t.feasible = ok;
            // under a budget: fastest feasible point (then least memory); under a target: least memory
            // (then fastest); with nothing feasible: the point closest to the constraint
            bool better;
            if (!have) better = true;
            else if (ok != (best.feasible != 0)) better = ok;
            else if (ok) {
                better = memory_budget_bytes
                             ? (t.sim.step_ms < best.sim.step_ms || (t.sim.step_ms == best.sim.step_ms && t.sim.weight_memory_bytes < best.sim.weight_memory_bytes))
                             : (t.sim.weight_memory_bytes < best.sim.weight_memory_bytes || (t.sim.weight_memory_bytes == best.sim.weight_memory_bytes && t.sim.step_ms < best.sim.step_ms));
            } else {
                better = memory_budget_bytes ? t.sim.weight_memory_bytes < best.sim.weight_memory_bytes : t.sim.step_ms < best.sim.step_ms;
            }
            if (better) { best = t; have = true; }
        }
    }
    *out = best;
    return CF_OK;
}

}  // extern "C"
