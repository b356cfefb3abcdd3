// bf16 MFMA GEMM for the block's linear layers (App. B: the projection and MLP terms):
//   out[m, n] = epilogue( sum_k A[m, k] * W[n, k] + bias[n] ),  fp32 accumulation.
// A is the activation matrix [M, K] (row-major, bf16); W is a linear weight stored
// [out_features, in_features] inside the block's weight blob, so both operands are
// K-contiguous and one launch can cover any panel [n0, n1) of output features -- the unit
// in which streamed weights become usable chunk by chunk (Sec. 3.2).
//
// Tiling: a workgroup of 4 waves owns a BM x BN output tile; each wave owns a
// (BM/2) x (BN/2) quadrant built from 32x32x16 bf16 MFMAs.  The MFMA "A" operand is the
// weight fragment and the "B" operand the activation fragment, so an accumulator lane holds
// one token row and 4 consecutive output features per register quad: epilogues then load
// bias/gate and store results 4 features at a time.  K is consumed in slabs of 64 that are
// copied global -> LDS directly (no register staging), double-buffered; 16-byte chunks of each
// 128-byte LDS row are XOR-swizzled so that the fragment reads of consecutive rows spread over
// all banks.  The k-steps are software-pipelined: LDS fragment reads of step s+1 and the
// slab hand-over barrier run behind the MFMAs of step s.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace {

constexpr int EPI_SPLIT_GELU_ERF = 2;  // kernel variant of EPI_SPLIT_GELU with the erf form of the activation
constexpr int BK = 64;                 // K slab (bf16 elements) = 128 bytes per LDS row
constexpr int STAGES = 2;              // slabs resident in LDS: one being multiplied, one in flight
constexpr int ROWB = BK * 2;           // bytes per LDS row
constexpr int CHUNKS = BK / 8;         // 16-byte chunks per LDS row
constexpr int KSTEPS = BK / 16;        // MFMA k-steps per slab

// slot of chunk c in row `row` is c ^ swz(row): conflict-free for 16-byte fragment reads of
// consecutive rows on a 32-bank (8 lanes per phase) as well as a 64-bank (16 lanes) LDS
__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 7) ^ ((row & 1) << 2); }

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at lds + 16*l
// (`lds` must be wave-uniform).
__device__ __forceinline__ void lds_load16(const void* gptr, void* lds) {
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gptr,
                                     (void __attribute__((address_space(3)))*)lds, 16, 0, 0);
}

// The same through a buffer resource: the address is base + voff (per lane) + soff (uniform), and
// lanes whose offset lies past the resource's size fetch zeros, which takes care of ragged tile
// edges.  The memory pipeline takes these a little faster than loads with a 64-bit address per lane.
__device__ __forceinline__ void lds_bload16(__amdgpu_buffer_rsrc_t rsrc, uint32_t voff, uint32_t soff, void* lds) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (void __attribute__((address_space(3)))*)lds, 16, voff, soff, 0, 0);
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint64_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)(bytes > 0xffffffffull ? 0xffffffffu : (uint32_t)bytes), 0x00020000);
}

// Slab hand-over: this wave's global->LDS loads (the next slab) have landed and its LDS reads
// (the last fragments of the current slab) have returned; after the barrier that holds for the
// whole workgroup, so the next slab may be read and the current one overwritten.
__device__ __forceinline__ void slab_handover() {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// One workgroup's tile of one problem: workgroup `bid` of the `nblk` that problem owns.
template <int BM, int BN, int EPI>
__device__ __forceinline__ void gemm_tile_body(const GemmArgs& g, uint32_t bid, uint32_t nblk) {
    constexpr int WM = BM / 2, WN = BN / 2;        // wave quadrant
    constexpr int MT = WM / 32, NT = WN / 32;      // 32x32 MFMA tiles per wave
    constexpr int A_LOADS = BM * CHUNKS / 256;     // 16-byte global loads per thread per slab
    constexpr int W_LOADS = BN * CHUNKS / 256;
    constexpr int RPL = 1024 / ROWB;               // LDS rows written by one wave-load
    constexpr int A_STAGE = BM * ROWB, W_STAGE = BN * ROWB;

    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* const sA = smem;                         // [STAGES][BM][ROWB] activations
    char* const sW = smem + STAGES * A_STAGE;      // [STAGES][BN][ROWB] weights

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN;
    const int li = lane & 31, lg = lane >> 5;

    // logical tile: XCD-contiguous id, then groups of GM row-tiles walked feature-tile-major
    const int tiles_m = (g.M + BM - 1) / BM;
    const int tiles_n = (g.n1 - g.n0 + BN - 1) / BN;
    const uint32_t lid = xcd_contiguous_id(bid, nblk);
    // row-tile groups of about 8, all of one size: a short last group would walk every weight tile once more
    const int n_groups = max(1, (tiles_m + 4) / 8);
    const int GM = (tiles_m + n_groups - 1) / n_groups;
    const int group = lid / (GM * tiles_n);
    const int first_m = group * GM;
    const int gsz = min(tiles_m - first_m, GM);
    const int tm = first_m + (lid % (GM * tiles_n)) % gsz;
    const int tn = (lid % (GM * tiles_n)) / gsz;
    const int m0 = tm * BM;
    const int n0 = g.n0 + tn * BN;

    // Slab copies go global -> LDS directly (no register staging).  One such load writes the
    // wave's 64 x 16 bytes to consecutive LDS addresses, i.e. RPL rows; which 16-byte chunk of
    // its row a lane fetches is chosen so that the chunk lands in its swizzled slot.
    const int uw = __builtin_amdgcn_readfirstlane(wave);
    uint32_t a_voff[A_LOADS], w_voff[W_LOADS];   // byte offsets from the tile's first row
    uint64_t w_src[W_LOADS];                     // blob offsets, for the tile that holds the resident/streamed split
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
        const int row = (j * 4 + uw) * RPL + lane / CHUNKS;
        const int c = (lane % CHUNKS) ^ swz(row);
        a_voff[j] = (uint32_t)row * (uint32_t)g.lda * 2u + c * 16;
    }
#pragma unroll
    for (int j = 0; j < W_LOADS; ++j) {
        const int row = (j * 4 + uw) * RPL + lane / CHUNKS;
        const int c = (lane % CHUNKS) ^ swz(row);
        w_voff[j] = (uint32_t)row * (uint32_t)g.K * 2u + c * 16;
        w_src[j] = g.w_off + ((uint64_t)min(n0 + row, g.N - 1) * g.K + c * 8) * 2;
    }
    // does the byte where the blob switches buffers fall inside this tile's weight rows?
    const uint64_t t_begin = g.w_off + (uint64_t)n0 * g.K * 2, t_end = g.w_off + (uint64_t)min(n0 + BN, g.N) * g.K * 2;
    const bool straddle = g.W.split > t_begin && g.W.split < t_end;
    // resources that end with the tile's last valid row: the rows of a ragged tile beyond it read zeros
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(g.A + (size_t)m0 * g.lda, ((uint64_t)(g.M - 1 - m0) * g.lda + g.K) * 2);
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(wv_ptr(g.W, t_begin), t_end - t_begin);

    floatx16 acc[NT][MT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // LDS byte offsets of this lane's fragment rows (row*ROWB) and their swizzle keys
    int a_off[MT], a_key[MT], w_off[NT], w_key[NT];
#pragma unroll
    for (int j = 0; j < MT; ++j) { const int row = wm0 + j * 32 + li; a_off[j] = row * ROWB; a_key[j] = swz(row); }
#pragma unroll
    for (int i = 0; i < NT; ++i) { const int row = wn0 + i * 32 + li; w_off[i] = row * ROWB; w_key[i] = swz(row); }

    const int KT = g.K / BK;
    bf16x8 fa[2][MT], fw[2][NT];

    // slab kt_ -> stage kt_&1
    auto issue_slab = [&](auto slow, int kt_) {
        const int k0 = kt_ * BK * 2, st = kt_ & 1;
        char* dA = sA + st * A_STAGE + uw * 1024;
        char* dW = sW + st * W_STAGE + uw * 1024;
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) lds_bload16(a_rsrc, a_voff[j], k0, dA + j * 4096);
#pragma unroll
        for (int j = 0; j < W_LOADS; ++j) {
            if (decltype(slow)::value) lds_load16(wv_ptr(g.W, w_src[j] + k0), dW + j * 4096);
            else lds_bload16(w_rsrc, w_voff[j], k0, dW + j * 4096);
        }
    };
    auto issue_one = [&](auto slow, int kt_, int q) {        // q-th load of slab kt_ (A loads first)
        const int k0 = kt_ * BK * 2, st = kt_ & 1;
        if (q < A_LOADS) {
            lds_bload16(a_rsrc, a_voff[q], k0, sA + st * A_STAGE + uw * 1024 + q * 4096);
        } else if (q < A_LOADS + W_LOADS) {
            const int j = q - A_LOADS;
            if (decltype(slow)::value) lds_load16(wv_ptr(g.W, w_src[j] + k0), sW + st * W_STAGE + uw * 1024 + j * 4096);
            else lds_bload16(w_rsrc, w_voff[j], k0, sW + st * W_STAGE + uw * 1024 + j * 4096);
        }
    };
    auto load_frags = [&](int buf, const char* cA, const char* cW, int kk) {
        const int c = kk * 2 + lg;
#pragma unroll
        for (int j = 0; j < MT; ++j) fa[buf][j] = *(const bf16x8*)(cA + a_off[j] + ((c ^ a_key[j]) << 4));
#pragma unroll
        for (int i = 0; i < NT; ++i) fw[buf][i] = *(const bf16x8*)(cW + w_off[i] + ((c ^ w_key[i]) << 4));
    };
    // One slab = KSTEPS k-steps, software-pipelined: the fragments of step s+1 are read from LDS
    // while the MFMAs of step s run.  The hand-over to the next slab sits before the slab's last
    // step: its barrier, the first fragment reads of the next slab and the issue of the slab after
    // that all hide behind that step's MFMAs.
    auto slab = [&](auto slow, auto handover, auto issue, int kt) {
        const char* cA = sA + (kt & 1) * A_STAGE;
        const char* cW = sW + (kt & 1) * W_STAGE;
        const char* nA = sA + ((kt + 1) & 1) * A_STAGE;
        const char* nW = sW + ((kt + 1) & 1) * W_STAGE;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const int cur = kk & 1, nxt = cur ^ 1;
            const bool last = kk + 1 == KSTEPS;
            if (!last) {
                load_frags(nxt, cA, cW, kk + 1);
            } else if (decltype(handover)::value) {
                __builtin_amdgcn_sched_barrier(0);     // keep the previous step's MFMAs above the barrier
                slab_handover();                       // slab kt+1 landed; slab kt fully read
                __builtin_amdgcn_sched_barrier(0);
                load_frags(nxt, nA, nW, 0);
            }
            if (last && decltype(issue)::value) {
                // the loads of slab kt+2 go out between this step's MFMAs, in this order
                constexpr int LPM = (A_LOADS + W_LOADS + MT * NT - 1) / (MT * NT);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < MT * NT; ++q) {
                    acc[q / MT][q % MT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[cur][q / MT], fa[cur][q % MT],
                                                                                  acc[q / MT][q % MT], 0, 0, 0);
#pragma unroll
                    for (int u = 0; u < LPM; ++u) issue_one(slow, kt + 2, q * LPM + u);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int i = 0; i < NT; ++i)
#pragma unroll
                    for (int j = 0; j < MT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[cur][i], fa[cur][j], acc[i][j], 0, 0, 0);
                if (!last || decltype(handover)::value) {
                    // fragment reads go out two per MFMA at the head of the step
#pragma unroll
                    for (int q = 0; q < (MT + NT) / 2; ++q) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, MT * NT - (MT + NT) / 2, 0);
                }
            }
        }
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    auto run = [&](auto slow) {
        issue_slab(slow, 0);
        slab_handover();
        if (KT > 1) issue_slab(slow, 1);
        load_frags(0, sA, sW, 0);
        int kt = 0;
        for (; kt + 2 < KT; ++kt) slab(slow, T_{}, T_{}, kt);
        if (kt + 1 < KT) { slab(slow, T_{}, F_{}, kt); ++kt; }
        slab(slow, F_{}, F_{}, kt);
    };
    if (straddle) run(T_{}); else run(F_{});

    // ---- epilogue.  In the accumulators a lane owns one token row and 4 consecutive features per
    // register quad.  Bias / GELU / gate are applied there, then each wave transposes its quadrant
    // through its own slice of LDS so that global stores are 16 bytes per lane with 16 (or 8)
    // consecutive lanes covering one contiguous row segment.
    constexpr bool OUT_BF16 = (EPI != EPI_GATE_RESID);
    constexpr bool ACT_ERF = (EPI == EPI_SPLIT_GELU_ERF);
    constexpr int PASSES = OUT_BF16 ? 1 : 2;               // fp32 rows are staged in two column halves
    constexpr int NTP = NT / PASSES;                       // 32-column tiles per pass
    constexpr int ELT = OUT_BF16 ? 2 : 4;
    constexpr int RB = NTP * 32 * ELT;                     // staged row bytes (= WN * 2 either way)
    constexpr int PITCH = RB + (OUT_BF16 ? 16 : 32);       // padded: conflict-free quad writes
    constexpr int CPR = RB / 16, RPI = 64 / CPR;           // 16-byte chunks per row, rows per store
    static_assert(4 * WM * PITCH <= 160 * 1024, "staging exceeds LDS");
    {   // the epilogue is a scope of its own: its lane coordinates shadow the main loop's
        // lane coordinates are derived afresh (lane from the wave's bit count, wave from its scalar copy)
        // rather than kept in vector registers across the main loop
        const int lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)), wave = uw;
        const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN;
        const int li = lane & 31, lg = lane >> 5;
        // Bias of the wave's features, in accumulator order: 4 consecutive features per (feature tile, register
        // quad).  Fetched in one go: taken one by one in the epilogue, each would cost a memory round trip.
        uint32x2 bias_raw[NT][4];
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int vb = 0; vb < 4; ++vb) bias_raw[i][vb] = uint32x2{0u, 0u};
        if (g.has_bias) {
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int vb = 0; vb < 4; ++vb) {
                    const int n = min(n0 + wn0 + i * 32 + vb * 8 + lg * 4, g.N - 4);
                    bias_raw[i][vb] = *(const uint32x2*)wv_ptr(g.W, g.bias_off + 2ull * n);
                }
        }
        slab_handover();                       // every wave is done reading the slabs; the bias loads flew meanwhile
        char* const stg = smem + wave * (WM * PITCH);
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
#pragma unroll
            for (int ii = 0; ii < NTP; ++ii) {
                const int i = p * NTP + ii;
#pragma unroll
                for (int vb = 0; vb < 4; ++vb) {
                    const int n = min(n0 + wn0 + i * 32 + vb * 8 + lg * 4, g.N - 4);
                    const uint32x2 bb = bias_raw[i][vb];
                    const float b[4] = {__uint_as_float(bb.x << 16), __uint_as_float(bb.x & 0xffff0000u),
                                        __uint_as_float(bb.y << 16), __uint_as_float(bb.y & 0xffff0000u)};
                    const bool act = OUT_BF16 && n >= g.n_split;
#pragma unroll
                    for (int j = 0; j < MT; ++j) {
                        float v[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][vb * 4 + e] + b[e];
                        char* dst = stg + (j * 32 + li) * PITCH + (ii * 32 + vb * 8 + lg * 4) * ELT;
                        if (OUT_BF16) {
                            if (act) {
#pragma unroll
                                for (int e = 0; e < 4; ++e) v[e] = ACT_ERF ? gelu_erf_f32(v[e]) : gelu_tanh_f32(v[e]);
                            }
                            bf16x4 o;
#pragma unroll
                            for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
                            *(bf16x4*)dst = o;
                        } else {
                            *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
                        }
                    }
                }
            }
            // coalesced write-out of this pass
            const int col = (lane % CPR) * (16 / ELT);                         // first column of the lane's chunk
            const int n = n0 + wn0 + p * (NTP * 32) + col;
            if constexpr (OUT_BF16) {
#pragma unroll
                for (int r = 0; r < WM / RPI; ++r) {
                    const int row = r * RPI + lane / CPR;
                    const int m = m0 + wm0 + row;
                    const uint4 val = *(const uint4*)(stg + row * PITCH + (lane % CPR) * 16);
                    if (m < g.M && n < g.n1) {
                        bf16* dst = n < g.n_split ? g.out0 + (size_t)m * g.ld0 + n
                                                  : g.out1 + (size_t)m * g.ld1 + g.col1_off + (n - g.n_split);
                        *(uint4*)dst = val;
                    }
                }
            } else {
                // y = resid + gate * (...), the product rounded before the sum; the gate belongs to the row's
                // sample.  The residual rows of UB stores are fetched together: taken one by one, each store
                // would wait out a memory round trip of its own.  Lanes outside the problem read a valid
                // address (row M-1, column 0) and store nothing.
                constexpr int UB = 8;
                static_assert((WM / RPI) % UB == 0, "write-out batches");
                const bool n_ok = n < g.n1;
                const int nc = n_ok ? n : 0;
                const bool has_gate = g.gate != nullptr;
                const float* const gate_p = has_gate ? g.gate : g.resid;       // a readable address either way
                const long gate_bs = has_gate ? g.gate_bs : 0;
                auto write_out = [&](auto per_sample) {
                    constexpr bool PS = decltype(per_sample)::value;
                    floatx4 gate_c = {1.f, 1.f, 1.f, 1.f};
                    if (!PS && has_gate) gate_c = *(const floatx4*)(gate_p + nc);
#pragma unroll
                    for (int r0 = 0; r0 < WM / RPI; r0 += UB) {
                        floatx4 rr[UB], gt[UB];                // native vectors: arrays of them stay in registers
                        size_t y_off[UB];
                        bool ok[UB];
#pragma unroll
                        for (int u = 0; u < UB; ++u) {
                            const int row = (r0 + u) * RPI + lane / CPR;
                            const int m = m0 + wm0 + row;
                            ok[u] = n_ok && m < g.M;
                            const int mm = min(m, g.M - 1);
                            int b = 0, i = mm;
                            if (PS) { b = mm / g.rows_per_sample; i = mm - b * g.rows_per_sample; }
                            rr[u] = *(const floatx4*)(g.resid + (size_t)b * g.resid_bs + (size_t)i * g.ldy + nc);
                            if (PS) {
                                const floatx4 t = *(const floatx4*)(gate_p + (size_t)b * gate_bs + nc);
                                gt[u] = has_gate ? t : gate_c;
                            } else {
                                gt[u] = gate_c;
                            }
                            y_off[u] = (size_t)b * g.y_bs + (size_t)i * g.ldy + nc;
                        }
#pragma unroll
                        for (int u = 0; u < UB; ++u) {
                            const int row = (r0 + u) * RPI + lane / CPR;
                            const floatx4 val = *(const floatx4*)(stg + row * PITCH + (lane % CPR) * 16);
                            floatx4 o;
#pragma unroll
                            for (int e = 0; e < 4; ++e) o[e] = __fadd_rn(rr[u][e], __fmul_rn(gt[u][e], val[e]));
                            if (ok[u]) *(floatx4*)(g.y + y_off[u]) = o;
                        }
                    }
                };
                if (g.rows_per_sample) write_out(std::true_type{}); else write_out(std::false_type{});
            }
        }
    }
}

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs g) {
    gemm_tile_body<BM, BN, EPI>(g, blockIdx.x, gridDim.x);
}

// Two independent problems of one tile shape and epilogue in one launch (the text and image streams
// of a double-stream block, App. B): a small problem's workgroups ride along with the large one's
// instead of holding the chip for the length of their K loop.  The first problem's share of the grid
// is padded to a multiple of 8 so that both keep the block-index-to-XCD correspondence.
struct GemmPair {
    GemmArgs g[2];
    uint32_t tiles0, tiles0_pad;
};
template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_pair_kernel(GemmPair p) {
    if (blockIdx.x < p.tiles0) gemm_tile_body<BM, BN, EPI>(p.g[0], blockIdx.x, p.tiles0);
    else if (blockIdx.x >= p.tiles0_pad) gemm_tile_body<BM, BN, EPI>(p.g[1], blockIdx.x - p.tiles0_pad, gridDim.x - p.tiles0_pad);
}

template <int BM, int BN, int EPI>
size_t gemm_smem() {
    const size_t stage_bytes = (size_t)STAGES * (BM + BN) * ROWB;
    const size_t epi_bytes = 4ull * (BM / 2) * (BN + (EPI != EPI_GATE_RESID ? 16 : 32));   // 4 x WM x PITCH
    return stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
}

template <int BM, int BN, int EPI>
hipError_t launch(const GemmArgs& g, hipStream_t s) {
    const int tiles_m = (g.M + BM - 1) / BM;
    const int tiles_n = (g.n1 - g.n0 + BN - 1) / BN;
    const size_t smem = gemm_smem<BM, BN, EPI>();
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_bf16_kernel<BM, BN, EPI>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, EPI>), dim3(tiles_m * tiles_n), dim3(256), smem, s, g);
    return hipGetLastError();
}

template <int BM, int BN, int EPI>
hipError_t launch_pair(const GemmArgs& g0, const GemmArgs& g1, hipStream_t s) {
    auto tiles = [](const GemmArgs& g) { return (uint32_t)(((g.M + BM - 1) / BM) * ((g.n1 - g.n0 + BN - 1) / BN)); };
    GemmPair p;
    p.g[0] = g0;
    p.g[1] = g1;
    p.tiles0 = tiles(g0);
    p.tiles0_pad = (p.tiles0 + 7u) & ~7u;
    const size_t smem = gemm_smem<BM, BN, EPI>();
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_pair_kernel<BM, BN, EPI>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((gemm_pair_kernel<BM, BN, EPI>), dim3(p.tiles0_pad + tiles(g1)), dim3(256), smem, s, p);
    return hipGetLastError();
}

}  // namespace

const char* gemm_check(const GemmArgs& g) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return "gemm: empty shape";
    if (g.K % 64) return "gemm: K must be a multiple of 64";
    if (g.N % 8) return "gemm: N must be a multiple of 8";
    if (g.n0 < 0 || g.n1 > g.N || g.n0 >= g.n1 || (g.n0 % 8) || (g.n1 % 8)) return "gemm: bad feature panel";
    if (g.lda < g.K || (g.lda % 8)) return "gemm: lda must be >= K and a multiple of 8";
    if ((uint64_t)g.lda * 512 >= (1ull << 32)) return "gemm: lda too large for 32-bit offsets inside a tile";
    if ((uint64_t)g.M * g.lda * 2 >= (1ull << 32)) return "gemm: activations beyond 4 GiB (32-bit buffer range)";
    if ((g.w_off % 16) || (g.has_bias && (g.bias_off % 16))) return "gemm: weight/bias offsets must be 16-byte aligned";
    if (((uintptr_t)g.A) % 16) return "gemm: A must be 16-byte aligned";
    if (g.epi == EPI_SPLIT_GELU) {
        if (g.n_split % 8) return "gemm: n_split must be a multiple of 8";
        if (g.n_split > 0 && (!g.out0 || (g.ld0 % 8) || ((uintptr_t)g.out0 % 16))) return "gemm: out0 must be 16-byte aligned with ld0 a multiple of 8";
        if (g.n_split < g.N && (!g.out1 || (g.ld1 % 8) || (g.col1_off % 8) || ((uintptr_t)g.out1 % 16)))
            return "gemm: out1 must be 16-byte aligned with ld1 and col1_off multiples of 8";
    } else if (g.epi == EPI_GATE_RESID) {
        if (!g.resid || !g.y || (g.ldy % 4) || ((uintptr_t)g.y % 16) || ((uintptr_t)g.resid % 16)) return "gemm: bad residual/output";
        if (g.gate && ((uintptr_t)g.gate % 16)) return "gemm: gate must be 16-byte aligned";
        if (g.rows_per_sample < 0 || (g.rows_per_sample && g.M % g.rows_per_sample)) return "gemm: M must be whole samples";
        if (g.rows_per_sample && ((g.gate_bs % 4) || (g.resid_bs % 4) || (g.y_bs % 4) || g.gate_bs < 0 || g.resid_bs < 0 || g.y_bs < 0))
            return "gemm: sample strides must be non-negative multiples of 4 elements";
    } else {
        return "gemm: unknown epilogue";
    }
    return nullptr;
}

// Tile shape for a launch: 0 = 256x256, 1 = 128x128.  The big tile has the best arithmetic
// intensity but needs enough tiles to cover the 256 CUs; estimated cost = rounds x tile area /
// relative efficiency of the shape (128x128 runs two workgroups per CU).  A 256-token x 128-feature
// tile looked better than 128x128 with operands hot in the last-level cache but was the slowest of
// the three inside a block, where every weight byte is read once, cold; it is not built.
namespace {
// cost of a launch over n output features in units of one round of 256x256 tiles on all CUs
void tile_costs(int M, long n, double* c256, double* c128) {
    const long m256 = (M + 255) / 256, m128 = (M + 127) / 128;
    const long n256 = (n + 255) / 256, n128 = (n + 127) / 128;
    auto rounds = [](long tiles, long slots) { return (double)((tiles + slots - 1) / slots); };
    *c256 = rounds(m256 * n256, 256) * 1.0;
    *c128 = rounds(m128 * n128, 512) * 2.0 * 0.25 / 0.65;
}
}  // namespace

int gemm_tile(const GemmArgs& g) {
    double c256, c128;
    tile_costs(g.M, g.n1 - g.n0, &c256, &c128);
    return c256 <= c128 ? 0 : 1;
}

// How well a launch over n output features uses the chip: work in rounds of 256x256 tiles divided
// by the estimated cost of the tile shape gemm_tile would pick (1 = whole rounds of the big tile).
double gemm_fill(int M, int n) {
    double c256, c128;
    tile_costs(M, n, &c256, &c128);
    const double work = (double)((M + 255) / 256) * (double)((n + 255) / 256) / 256.0;
    return work / std::min(c256, c128);
}

// Diagnostic: nothing but 32x32x16 bf16 MFMAs on registers, one wave per SIMD on every CU, four
// independent accumulators per wave.  Its rate is what the matrix cores sustain at the clock the
// chip settles to under this load (the published peak assumes the maximum clock).  The clock depends
// on what the operands look like: `random_operands` = 0 feeds the same small values to every MFMA,
// 1 feeds sixteen different pairs of pseudo-random fragments spread like N(0,1) data, as a GEMM does.
namespace {
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, int random_operands, float* out) {
    bf16x8 a[4], b[4];
    uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            h = h * 1664525u + 1013904223u;
            const float u = (float)(h >> 8) * (1.0f / 16777216.0f);          // [0, 1)
            h = h * 1664525u + 1013904223u;
            const float w = (float)(h >> 8) * (1.0f / 16777216.0f);
            a[i][e] = random_operands ? (bf16)(3.46f * (u - 0.5f)) : (bf16)(0.001f * (threadIdx.x + e));   // unit variance
            b[i][e] = random_operands ? (bf16)(3.46f * (w - 0.5f)) : (bf16)(0.002f * (e + 1));
        }
    floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int q = 0; q < 16; ++q)
            acc[q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[random_operands ? (q & 3) : 0], b[random_operands ? (q >> 2) : 0],
                                                                 acc[q & 3], 0, 0, 0);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}
}  // namespace

// `out` holds 256 * 256 floats; FLOPs of a launch = 256 workgroups x 4 waves x iters x 16 MFMAs x 32768
hipError_t mfma_rate_launch(int iters, int random_operands, float* out, hipStream_t s) {
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(256), dim3(256), 0, s, iters, random_operands, out);
    return hipGetLastError();
}

// Diagnostic: what the matrix cores deliver when a wave's MFMAs share the SIMD with the other work a kernel
// has to issue -- LDS fragment reads (ds_read_b128 through a ring of four fragments) and ordinary / transcendental
// VALU instructions.  Per 16 MFMAs (four independent accumulators) a wave issues READS16 fragment reads,
// 16 * VALU fused multiply-adds and 16 * EXPS exp2's; `waves` waves per workgroup, one workgroup per CU.
// No global memory traffic, no barriers: the rate is the ceiling of an instruction mix, whatever the schedule.
namespace {
template <int READS16, int VALU, int EXPS>
__global__ void mix_rate_kernel(int iters, float* out) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef __attribute__((address_space(3))) const volatile bf16x8 lds_frag;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nthr = blockDim.x;
    for (int i = threadIdx.x; i < 65536 / 4; i += nthr) {           // pairs of small bf16 values
        const bf16 lo = (bf16)(0.01f * (i % 37 - 18)), hi = (bf16)(0.01f * (i % 41 - 20));
        ((uint32_t*)smem)[i] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
    }
    __syncthreads();
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[i][e] = (bf16)(0.01f * ((lane * 7 + e * 3 + i) % 97 - 48));
            b[i][e] = (bf16)(0.02f * ((lane * 5 + e + i * 11) % 89 - 44));
        }
    floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    float vv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) vv[i] = 0.5f + 0.01f * (lane + i);
    const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + ((wave * 4096) & 0xffff) + lane * 16;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            acc[q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[q & 3], b[q >> 2], acc[q & 3], 0, 0, 0);
            if (READS16 > 0 && (q % (16 / (READS16 > 0 ? READS16 : 1))) == 0)
                a[q & 3] = *(lds_frag*)(uintptr_t)(base + ((q * 1024 + it * 64) & 0x3fff));     // the fragment four slots ahead
#pragma unroll
            for (int u = 0; u < VALU; ++u) vv[(q * VALU + u) & 7] = __builtin_fmaf(vv[(q * VALU + u) & 7], 0.9999f, 0.0001f);   // -> 1
#pragma unroll
            for (int u = 0; u < EXPS; ++u) vv[(q + 3) & 7] = __builtin_amdgcn_exp2f(-vv[(q + 3) & 7]);                       // stays in (0, 1]
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
#pragma unroll
    for (int i = 0; i < 8; ++i) s += vv[i];
    out[blockIdx.x * nthr + threadIdx.x] = s;
}

template <int READS16, int VALU, int EXPS>
hipError_t mix_rate_go(int iters, int waves, float* out, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)mix_rate_kernel<READS16, VALU, EXPS>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((mix_rate_kernel<READS16, VALU, EXPS>), dim3(256), dim3(64 * waves), 65536, s, iters, out);
    return hipGetLastError();
}
}  // namespace

// `out`: 256 * 64 * waves floats.  FLOPs of a launch = 256 * waves * iters * 16 * 32768.  Supported mixes:
// reads16 in {0, 8, 16}, valu in {0, 2, 4}, exps in {0, 1}, waves in {4, 8}.
hipError_t mix_rate_launch(int iters, int waves, int reads16, int valu, int exps, float* out, hipStream_t s) {
    if (waves != 4 && waves != 8) return hipErrorInvalidValue;
#define CF_MIX(R, V, E) if (reads16 == R && valu == V && exps == E) return mix_rate_go<R, V, E>(iters, waves, out, s);
    CF_MIX(0, 0, 0) CF_MIX(8, 0, 0) CF_MIX(16, 0, 0)
    CF_MIX(0, 2, 0) CF_MIX(0, 4, 0) CF_MIX(0, 2, 1) CF_MIX(0, 4, 1)
    CF_MIX(8, 2, 1) CF_MIX(8, 4, 1) CF_MIX(16, 2, 1) CF_MIX(16, 4, 1)
#undef CF_MIX
    return hipErrorInvalidValue;
}

hipError_t gemm_launch(const GemmArgs& g, hipStream_t s) {
    const int t = gemm_tile(g);
    // the erf form of the activation costs some forty VALU operations per element: it gets kernels
    // of its own rather than a run-time choice inside the tanh one
    if (g.epi == EPI_SPLIT_GELU && g.act_erf)
        return t == 0 ? launch<256, 256, EPI_SPLIT_GELU_ERF>(g, s) : launch<128, 128, EPI_SPLIT_GELU_ERF>(g, s);
    if (g.epi == EPI_SPLIT_GELU) return t == 0 ? launch<256, 256, EPI_SPLIT_GELU>(g, s) : launch<128, 128, EPI_SPLIT_GELU>(g, s);
    return t == 0 ? launch<256, 256, EPI_GATE_RESID>(g, s) : launch<128, 128, EPI_GATE_RESID>(g, s);
}

// Tile shape both problems of a pair run with, or -1 if they cannot share a launch (different
// epilogues).  Shapes that would pick different tiles alone take the larger problem's choice.
int gemm_pair_tile(const GemmArgs& g0, const GemmArgs& g1) {
    if (g0.epi != g1.epi || g0.act_erf != g1.act_erf) return -1;
    const GemmArgs& big = (double)g0.M * (g0.n1 - g0.n0) >= (double)g1.M * (g1.n1 - g1.n0) ? g0 : g1;
    return gemm_tile(big);
}

hipError_t gemm_launch_pair(const GemmArgs& g0, const GemmArgs& g1, hipStream_t s) {
    const int t = gemm_pair_tile(g0, g1);
    if (t < 0) return hipErrorInvalidValue;
    if (g0.epi == EPI_SPLIT_GELU && g0.act_erf)
        return t == 0 ? launch_pair<256, 256, EPI_SPLIT_GELU_ERF>(g0, g1, s) : launch_pair<128, 128, EPI_SPLIT_GELU_ERF>(g0, g1, s);
    if (g0.epi == EPI_SPLIT_GELU)
        return t == 0 ? launch_pair<256, 256, EPI_SPLIT_GELU>(g0, g1, s) : launch_pair<128, 128, EPI_SPLIT_GELU>(g0, g1, s);
    return t == 0 ? launch_pair<256, 256, EPI_GATE_RESID>(g0, g1, s) : launch_pair<128, 128, EPI_GATE_RESID>(g0, g1, s);
}
