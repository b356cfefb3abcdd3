// Full (non-causal, unmasked) softmax attention for the heads this rank owns, over the whole
// joint sequence (App. B: the 4*B*S^2*d term; Sec. 2.1: under Ulysses each rank attends over all
// N tokens for H/P heads).  Flash-style: the nq x nk score matrix is never materialised; keys
// and values stream through LDS in tiles of 64 keys with an online softmax.
//
// The kernel works on the transposed problem so that no data ever changes lanes between the
// two contractions:
//   S^T[key, query] = K . Q^T      (MFMA A = key rows from LDS,   B = query fragment in registers)
//   O^T[d,   query] = V^T . P^T    (MFMA A = V^T rows from LDS,   B = P^T built from S^T registers)
// With 32x32x16 MFMAs a lane owns ONE query column, so the softmax reference and the row sum are
// per-lane scalars and a rescale of O^T is a lane-uniform multiply.  The 32 key rows of each S^T tile
// are fed in an order that swaps bits 2 and 3 of the row index; the accumulator registers
// v=8a..8a+7 of lane group g then hold keys 16a+8g .. 16a+8g+7 in order, which is exactly the
// B-operand layout of the second contraction (8 consecutive k per lane), so P^T is a pure
// register repack.  V is kept transposed in HBM ([head, d, key]) so that its A-operand rows
// are contiguous 16-byte reads as well.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace {

// One wave-load: 64 lanes x 16 bytes from global memory straight into 1 KiB of consecutive LDS.
// The address is base + voff (per lane) + soff (uniform, advanced per tile); lanes whose offset
// lies past the resource's size fetch zeros, which takes care of the ragged last K tile.
__device__ __forceinline__ void lds_bload16(__amdgpu_buffer_rsrc_t rsrc, uint32_t voff, uint32_t soff, void* lds) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (void __attribute__((address_space(3)))*)lds, 16, voff, soff, 0, 0);
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint64_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)(bytes > 0xffffffffull ? 0xffffffffu : (uint32_t)bytes), 0x00020000);
}

constexpr int BKV = 64;    // keys per tile

__device__ __forceinline__ float max3f(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

// NW waves of 32 queries each per workgroup: 4 (two workgroups per CU), 7 or 8 (one per CU).
template <int HD, int NW>
__global__ __launch_bounds__(64 * NW, 2) void attn_fwd_kernel(AttnArgs a) {
    constexpr int BQ = 32 * NW;
    constexpr int KCH = HD / 8;                 // 16-byte chunks per K row
    constexpr int KROW = HD * 2;                // bytes per K row in LDS
    constexpr int KL = BKV * KCH / 64, VL = HD * 8 / 64;   // wave-loads (1 KiB each) per K / V^T tile
    constexpr int LPW = (KL + VL + NW - 1) / NW;           // wave-loads per wave per tile (round robin)
    constexpr int K_TILE = BKV * KROW, V_TILE = HD * 128;
    constexpr int DT = HD / 32;                 // 32-row tiles of O^T
    constexpr int KS = HD / 16;                 // k-steps of the first contraction

    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* const sK = smem;                      // [2][BKV][KROW]
    char* const sV = smem + 2 * K_TILE;         // [2][HD][128]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lj = lane & 31, lg = lane >> 5;

    const int nqt = (a.nq + BQ - 1) / BQ;
    const uint32_t lid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int h = lid / nqt, qt = lid % nqt;
    const int q0 = qt * BQ + wave * 32;

    // K swizzle: 256-byte rows (HD=128) rotate over 16 chunk slots, 128-byte rows over 8
    auto kswz = [](int key) { return HD == 128 ? (key & 15) : (((key >> 1) & 7) ^ ((key & 1) << 2)); };
    auto vswz = [](int row) { return ((row >> 1) & 7) ^ ((row & 1) << 2); };

    // ---- query fragments (B operand), resident in registers for the whole sweep
    bf16x8 qf[KS];
    {
        const int qr = min(q0 + lj, a.nq - 1);
        const bf16* qp = a.Q + ((size_t)h * a.nq + qr) * HD + lg * 8;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) qf[kk] = *(const bf16x8*)(qp + kk * 16);
    }

    // ---- tile copies go global -> LDS directly: one load writes the wave's 64 x 16 bytes to
    // consecutive LDS addresses (1 KiB = 1024/KROW key rows, or 8 V^T rows); the 16-byte chunk a
    // lane fetches is the one whose swizzled slot it fills.  Per-lane offsets are computed once; a
    // tile only advances the uniform offset, so the copies cost no vector instructions per tile.
    // Key rows past nk read zeros (their scores are masked below); V^T rows are padded to nk_pad.
    const int uw = __builtin_amdgcn_readfirstlane(wave);
    constexpr int K_RPL = 1024 / KROW;          // key rows per wave-load
    const __amdgpu_buffer_rsrc_t k_rsrc = make_rsrc(a.K + (size_t)h * a.nk * HD, (uint64_t)a.nk * KROW);
    const __amdgpu_buffer_rsrc_t v_rsrc = make_rsrc(a.Vt + (size_t)h * HD * a.nk_pad, (uint64_t)HD * a.nk_pad * 2);
    uint32_t t_voff[LPW];                       // wave-load j = jj * NW + wave: K loads first, then V^T
#pragma unroll
    for (int jj = 0; jj < LPW; ++jj) {
        const int j = jj * NW + uw;
        if (j < KL) {
            const int key = j * K_RPL + lane / KCH;
            t_voff[jj] = (uint32_t)key * KROW + (((lane % KCH) ^ kswz(key)) << 4);
        } else {
            const int row = min(j - KL, VL - 1) * 8 + (lane >> 3);
            t_voff[jj] = (uint32_t)row * (uint32_t)a.nk_pad * 2 + (((lane & 7) ^ vswz(row)) << 4);
        }
    }
    auto issue_tile = [&](int t, int buf) {
        const uint32_t k_soff = (uint32_t)t * (BKV * KROW), v_soff = (uint32_t)t * (BKV * 2);
#pragma unroll
        for (int jj = 0; jj < LPW; ++jj) {
            // with KL a multiple of NW a wave-load's role is known at compile time
            constexpr bool kStatic = KL % NW == 0;
            const int j = jj * NW + uw;         // wave-uniform
            const bool is_k = kStatic ? jj < KL / NW : j < KL;
            if (is_k)
                lds_bload16(k_rsrc, t_voff[jj], k_soff, sK + buf * K_TILE + j * 1024);
            else if (kStatic || j < KL + VL)
                lds_bload16(v_rsrc, t_voff[jj], v_soff, sV + buf * V_TILE + (j - KL) * 1024);
        }
    };

    floatx16 o[DT];
    float mc, l_run;                            // reference of the exponentials (base-2 units), row sum
    const float c2 = a.scale * 1.4426950408889634f;   // logits in base-2 units

    // key row fed to MFMA row i: swap bits 2 and 3 of i
    const int krow = (lj & 0x13) | ((lj & 4) << 1) | ((lj & 8) >> 1);

    const int NT = (a.nk + BKV - 1) / BKV;
    int out_of_range = 0;                       // wave-uniform: a fast tile met scores it could not take

    // One tile.  The LDS buffer is a compile-time constant so that fragment addresses are a per-lane
    // register plus an immediate.
    //
    // Softmax is invariant to the reference its exponentials are taken against, as long as numerator and
    // denominator share it; magnitudes only have to stay inside the fp32 / bf16 range, whose relative
    // precision does not depend on scale.  A tracking tile does what online softmax usually does: take
    // the tile's maximum, move the reference there, rescale O^T and the row sum.  A fast tile takes no
    // maximum: it forms P^T = exp2(s * c2 - mc) against the reference it inherits (one FMA, one exp2 and
    // half a conversion per score) and looks at the row sums afterwards.  A query whose 64 values add
    // up to 2^20 or more has its reference, O^T and row sum shifted by a whole power of two (exact); if
    // they add up to 2^64 or more, or to no number (exp2 overflowed), the tile is declared out of range:
    // nothing is repaired on the spot, the workgroup repeats the whole sweep with tracking tiles.
    auto tile = [&](int t, auto buf_c, auto tracking_c) __attribute__((always_inline)) {
        constexpr int buf = decltype(buf_c)::value;
        constexpr bool tracking = decltype(tracking_c)::value;
        if (t + 1 < NT) issue_tile(t + 1, buf ^ 1);
        const char* cK = sK + buf * K_TILE;
        const char* cV = sV + buf * V_TILE;

        // ---- S^T = K . Q^T for 2 x 32 keys.  MFMA i handles key half (i & 1) and k-step (i >> 1), so
        // consecutive MFMAs hit different accumulators; K fragments run 4 reads ahead in a ring.
        // Register v of tile mt is key k0 + mt*32 + 16*(v/8) + 8*lg + v%8; keys past nk score -inf.
        floatx16 s[2];
        const int k0 = t * BKV;
        {
            bf16x8 kf[4];
            auto kfrag = [&](int i) {
                const int key = (i & 1) * 32 + krow, c = (i >> 1) * 2 + lg;
                return *(const bf16x8*)(cK + key * KROW + ((c ^ kswz(key)) << 4));
            };
#pragma unroll
            for (int i = 0; i < 4; ++i) kf[i] = kfrag(i);
#pragma unroll
            for (int i = 0; i < 2 * KS; ++i) {
                if (i < 2) {
                    floatx16 z;
#pragma unroll
                    for (int v = 0; v < 16; ++v) z[v] = 0.f;
                    s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i & 3], qf[i >> 1], z, 0, 0, 0);
                } else {
                    s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i & 3], qf[i >> 1], s[i & 1], 0, 0, 0);
                }
                if (i + 4 < 2 * KS) kf[i & 3] = kfrag(i + 4);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
            for (int i = 0; i < 2 * KS - 4; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
        }
        if (k0 + BKV > a.nk) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = k0 + mt * 32 + 16 * (v >> 3) + 8 * lg + (v & 7);
                    if (key >= a.nk) s[mt][v] = -INFINITY;
                }
        }
        // first V^T fragments: issued now so that they land while the softmax runs
        bf16x8 vf[4];
        auto vfrag = [&](int i) {                   // i = ks * DT + d
            const int row = (i % DT) * 32 + lj, c = (i / DT) * 2 + lg;
            return *(const bf16x8*)(cV + row * 128 + ((c ^ vswz(row)) << 4));
        };
#pragma unroll
        for (int i = 0; i < 4; ++i) vf[i] = vfrag(i);
        // The softmax stays between two scheduling fences: in one region with the second contraction the
        // compiler threads the exponentials between its MFMAs, which measured 5 % slower than keeping
        // the three phases apart and leaving the overlap to the SIMD's other wave.
        __builtin_amdgcn_sched_barrier(0);

        if constexpr (tracking) {
            float mx;                                   // the lane's 32 scores: a tree of three-input maxima
            {
                float m3[11];
#pragma unroll
                for (int i = 0; i < 10; ++i) m3[i] = max3f(s[(3 * i) >> 4][(3 * i) & 15], s[(3 * i + 1) >> 4][(3 * i + 1) & 15], s[(3 * i + 2) >> 4][(3 * i + 2) & 15]);
                m3[10] = fmaxf(s[1][14], s[1][15]);
                const float a0 = max3f(m3[0], m3[1], m3[2]), a1 = max3f(m3[3], m3[4], m3[5]), a2 = max3f(m3[6], m3[7], m3[8]);
                mx = max3f(max3f(a0, a1, a2), m3[9], m3[10]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32));         // every tile holds a key below nk: mx is finite
            const float mc_new = fmaxf(mc, mx * c2);
            const float alpha = __builtin_amdgcn_exp2f(mc - mc_new);             // 0 from mc = -inf
            l_run *= alpha;
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[d][v] *= alpha;
            mc = mc_new;
        }

        // ---- P^T in bf16, in the B-operand layout of the second contraction (fragment ks = registers
        // 8*(ks&1).. of half ks>>1).  The row sum adds the rounded values in pairs (bf16 dot product with
        // (1, 1), fp32 accumulate): the weights the second contraction really applies to V.
        bf16x8 pf[4];
        float psum;
        {
            float ps[4] = {0.f, 0.f, 0.f, 0.f};           // four chains: a row sum is not one long dependency
            bf16x2 ones;
            ones[0] = (bf16)1.0f;
            ones[1] = (bf16)1.0f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    bf16x2 pp;
                    pp[0] = (bf16)__builtin_amdgcn_exp2f(fmaf(s[ks >> 1][8 * (ks & 1) + e], c2, -mc));
                    pp[1] = (bf16)__builtin_amdgcn_exp2f(fmaf(s[ks >> 1][8 * (ks & 1) + e + 1], c2, -mc));
                    pf[ks][e] = pp[0];
                    pf[ks][e + 1] = pp[1];
                    ps[(e >> 1) & 3] = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, ps[(e >> 1) & 3], false);
                }
            psum = (ps[0] + ps[1]) + (ps[2] + ps[3]);
        }
        l_run += psum;
        __builtin_amdgcn_sched_barrier(0);

        // ---- O^T += V^T . P^T: MFMA i handles k-step (i / DT) of 16 keys and d-tile (i % DT);
        // V^T fragments keep running 4 reads ahead
        {
#pragma unroll
            for (int i = 0; i < 4 * DT; ++i) {
                o[i % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i & 3], pf[i / DT], o[i % DT], 0, 0, 0);
                if (i + 4 < 4 * DT) vf[i & 3] = vfrag(i + 4);
            }
#pragma unroll
            for (int i = 0; i < 4 * DT - 4; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 1);
        }

        if constexpr (!tracking) {
            const float row = psum + __shfl_xor(psum, 32);
            if (__any(!(row < 1048576.0f))) {
                if (__any(!(row < 18446744073709551616.0f))) {
                    out_of_range = 1;
                } else {
                    // queries at or past 2^20: divide by 2^e, e = the sum's binary exponent; the others keep e = 0
                    const int e = row < 1048576.0f ? 0 : (int)(__float_as_uint(row) >> 23) - 127;
                    const float alpha = __uint_as_float((uint32_t)(127 - e) << 23);
                    mc += (float)e;
                    l_run *= alpha;
#pragma unroll
                    for (int d = 0; d < DT; ++d)
#pragma unroll
                        for (int v = 0; v < 16; ++v) o[d][v] *= alpha;
                }
            }
        }

        __syncthreads();                        // tile t+1 has landed, tile t may be overwritten
    };
    // One sweep over the keys: the first tile always tracks (it sets the reference), the others in pairs.
    auto sweep = [&](auto tracking_c) __attribute__((always_inline)) {
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[d][v] = 0.f;
        mc = -INFINITY;
        l_run = 0.f;
        issue_tile(0, 0);
        __syncthreads();                        // (waits for the LDS-DMA, then the barrier)
        tile(0, std::integral_constant<int, 0>{}, std::true_type{});
        for (int t = 1; t < NT; t += 2) {
            tile(t, std::integral_constant<int, 1>{}, tracking_c);
            if (t + 1 < NT) tile(t + 1, std::integral_constant<int, 0>{}, tracking_c);
        }
    };
    sweep(std::false_type{});
    // the K/V tiles are the workgroup's: if any wave met a tile out of range, all of them go again
    if (__syncthreads_or(out_of_range)) sweep(std::true_type{});

    // ---- normalise and store: lane = query, register quad = 4 consecutive d
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.0f / l_tot;
    const int q = q0 + lj;
    if (q < a.nq) {
        const int hps = a.hps ? a.hps : a.H;            // heads per sample of a batch
        const int b = h / hps, hh = h % hps;
        bf16* op;
        if (a.scatter) {
            // the second exchange by the stores themselves: this rank's positions go to the projection operand,
            // the others to the send buffer (in ascending position order, as the receiver expects them)
            const TokenMap& m = a.map;
            if (q >= m.pos0 && q < m.pos0 + m.len0) {
                op = a.dst0 + (size_t)b * a.bs0 + (size_t)(q - m.pos0) * a.ld + (a.h0 + hh) * HD;
            } else if (q >= m.pos1 && q < m.pos1 + m.len1) {
                op = a.dst1 + (size_t)b * a.bs1 + (size_t)(q - m.pos1) * a.ld + (a.h0 + hh) * HD;
            } else {
                const int ri = q - (q >= m.pos0 + m.len0 ? m.len0 : 0) - (q >= m.pos1 + m.len1 ? m.len1 : 0);
                op = a.send ? a.send + (size_t)b * a.send_bs + ((size_t)hh * (m.n_total - m.n_local) + ri) * HD : nullptr;
            }
        } else {
            op = a.O + (size_t)b * a.o_bs + (size_t)hh * a.o_hs + (size_t)q * a.o_qs;
        }
        if (op) {
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int vb = 0; vb < 4; ++vb) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (bf16)(o[d][vb * 4 + e] * inv);
                *(bf16x4*)(op + d * 32 + vb * 8 + lg * 4) = w;
            }
        }
    }
}

template <int HD, int NW>
hipError_t launch(const AttnArgs& a, hipStream_t s) {
    const size_t smem = 2 * (BKV * HD * 2 + HD * 128);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)attn_fwd_kernel<HD, NW>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int nqt = (a.nq + 32 * NW - 1) / (32 * NW);
    hipLaunchKernelGGL((attn_fwd_kernel<HD, NW>), dim3(nqt * a.H), dim3(64 * NW), smem, s, a);
    return hipGetLastError();
}

template <int HD>
hipError_t launch_nw(int nw, const AttnArgs& a, hipStream_t s) {
    switch (nw) {
        case 7: return launch<HD, 7>(a, s);
        case 8: return launch<HD, 8>(a, s);
        default: return launch<HD, 4>(a, s);
    }
}

}  // namespace

const char* attn_check(const AttnArgs& a) {
    if (a.hd != 64 && a.hd != 128) return "attention: head_dim must be 64 or 128";
    if (a.H <= 0 || a.nq <= 0 || a.nk <= 0) return "attention: empty shape";
    if (a.nk_pad % 64 || a.nk_pad < a.nk) return "attention: nk_pad must be a multiple of 64 covering nk";
    if ((uint64_t)a.nk_pad * a.hd * 2 >= (1ull << 32)) return "attention: a head's keys exceed the 4 GiB buffer range";
    if (!a.Q || !a.K || !a.Vt) return "attention: null operand";
    if (((uintptr_t)a.Q | (uintptr_t)a.K | (uintptr_t)a.Vt) % 16) return "attention: operands must be 16-byte aligned";
    if (a.scatter) {
        const TokenMap& m = a.map;
        if (!a.dst0 || (m.len1 > 0 && !a.dst1)) return "attention: scatter mode needs the projection operand";
        if (m.n_total != a.nq || m.len0 + m.len1 != m.n_local || m.pos0 < 0 || m.len0 < 0 || m.len1 < 0 ||
            m.pos0 + m.len0 > m.pos1 || m.pos1 + m.len1 > m.n_total)
            return "attention: scatter map must hold two ordered position ranges inside the query sequence";
        if ((((uintptr_t)a.dst0 | (uintptr_t)a.dst1 | (uintptr_t)a.send) % 8) || (a.ld % 4) || (a.bs0 % 4) || (a.bs1 % 4) || (a.send_bs % 4))
            return "attention: scatter targets must be 8-byte aligned";
        if (a.h0 < 0 || a.ld < (a.h0 + (a.hps ? a.hps : a.H)) * a.hd) return "attention: scatter columns exceed the operand's row";
    } else {
        if (!a.O) return "attention: null operand";
        if (((uintptr_t)a.O % 8) || (a.o_hs % 4) || (a.o_qs % 4) || (a.o_bs % 4)) return "attention: output must be 8-byte aligned";
    }
    if (a.hps < 0 || (a.hps && a.H % a.hps)) return "attention: H must be whole samples of hps heads";
    if ((long)((a.nq + 127) / 128) * a.H > 0x7fffffffL) return "attention: grid too large";
    return nullptr;
}

// Waves per workgroup.  A CU holds 8 waves of this kernel, as one workgroup of 7 or 8 or as two of 4, and
// runs its workgroups generation after generation; a generation takes about as long whether the chip is
// full of workgroups or holds a handful.  Estimated time, in units of one K/V tile of an 8-wave workgroup
// (fitted to sweeps of 8 to 1861 tiles on 12 to 24 heads):
//   8 waves: generations x (tiles + 2.5)           the fixed part is the prologue and epilogue nothing overlaps
//   7 waves: generations x (0.96 tiles + 9)        a little faster per tile (one SIMD holds a single wave), its
//                                                  tile copies dealt unevenly; never fewer generations than 8
//   4 waves: generations x (1.08 tiles + 0.5)      twice the tile copies per query, but one workgroup's fixed
//                                                  part hides behind the other's tiles, and a last generation
//                                                  of at most one workgroup per CU takes 0.55 of a full one
// Short sweeps (cross-attention to a few hundred keys) and grids that end on a half-empty generation go to
// 4; very long sweeps whose 7- and 8-wave grids need the same number of generations to 7; the rest to 8.
// Heights 5 and 6 were built once and never won: three SIMDs share the work of four.
int attn_waves(const AttnArgs& a) {
    // a grid that cannot even give every CU one 4-wave workgroup is spread as widely as possible
    if ((long)((a.nq + 127) / 128) * a.H <= 256) return 4;
    const double tiles = (double)((a.nk + BKV - 1) / BKV);
    auto items = [&](int nw) { return (long)((a.nq + 32 * nw - 1) / (32 * nw)) * a.H; };
    auto generations = [](long n, long slots) { return (double)((n + slots - 1) / slots); };
    const double c8 = generations(items(8), 256) * (tiles + 2.5);
    const double c7 = generations(items(7), 256) * (0.96 * tiles + 9.0);
    const long full4 = items(4) / 512, rest4 = items(4) % 512;
    const double c4 = ((double)full4 + (rest4 == 0 ? 0.0 : (rest4 <= 256 ? 0.55 : 1.0))) * (1.08 * tiles + 0.5);
    int best = 8;
    double best_cost = c8;
    if (c7 < best_cost - 1e-9) { best = 7; best_cost = c7; }
    if (c4 < best_cost - 1e-9) { best = 4; best_cost = c4; }
    return best;
}

hipError_t attn_launch(const AttnArgs& a, hipStream_t s) {
    const int nw = attn_waves(a);
    return a.hd == 128 ? launch_nw<128>(nw, a, s) : launch_nw<64>(nw, a, s);
}
