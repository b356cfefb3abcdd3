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
// 128-byte LDS row are XOR-swizzled so that the fragment reads of 16..32 consecutive rows
// spread over all banks.
#include "common.h"
#include "kernels.h"

namespace {

constexpr int BK = 64;                 // K slab (bf16 elements) = 128 bytes per LDS row
constexpr int CHUNKS = BK / 8;         // 16-byte chunks per LDS row

__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 7) ^ ((row & 1) << 2); }

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at lds + 16*l
// (`lds` must be wave-uniform).
__device__ __forceinline__ void lds_load16(const void* gptr, void* lds) {
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gptr,
                                     (void __attribute__((address_space(3)))*)lds, 16, 0, 0);
}

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs g) {
    constexpr int WM = BM / 2, WN = BN / 2;        // wave quadrant
    constexpr int MT = WM / 32, NT = WN / 32;      // 32x32 MFMA tiles per wave
    constexpr int A_LOADS = BM * CHUNKS / 256;     // 16-byte global loads per thread per slab
    constexpr int W_LOADS = BN * CHUNKS / 256;

    extern __shared__ __attribute__((aligned(16))) char smem[];
    // [2][BM][128 B] activations, then [2][BN][128 B] weights
    char* const sA = smem;
    char* const sW = smem + 2 * BM * 128;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN;
    const int li = lane & 31, lg = lane >> 5;

    // logical tile: XCD-contiguous id, then groups of GM row-tiles walked feature-tile-major
    const int tiles_m = (g.M + BM - 1) / BM;
    const int tiles_n = (g.n1 - g.n0 + BN - 1) / BN;
    const uint32_t lid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    constexpr int GM = 8;
    const int group = lid / (GM * tiles_n);
    const int first_m = group * GM;
    const int gsz = min(tiles_m - first_m, GM);
    const int tm = first_m + (lid % (GM * tiles_n)) % gsz;
    const int tn = (lid % (GM * tiles_n)) / gsz;
    const int m0 = tm * BM;
    const int n0 = g.n0 + tn * BN;

    // Slab copies go global -> LDS directly (no register staging).  One such load writes the
    // wave's 64 x 16 bytes to consecutive LDS addresses, i.e. 8 rows of 128 bytes; which 16-byte
    // chunk of its row a lane fetches is chosen so that the chunk lands in its swizzled slot.
    const int uw = __builtin_amdgcn_readfirstlane(wave);
    const bf16* a_src[A_LOADS];
    uint64_t w_src[W_LOADS];
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
        const int row = (j * 4 + uw) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ swz(row);
        a_src[j] = g.A + (size_t)min(m0 + row, g.M - 1) * g.lda + c * 8;
    }
#pragma unroll
    for (int j = 0; j < W_LOADS; ++j) {
        const int row = (j * 4 + uw) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ swz(row);
        w_src[j] = g.w_off + ((uint64_t)min(n0 + row, g.N - 1) * g.K + c * 8) * 2;
    }

    floatx16 acc[NT][MT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    auto issue_slab = [&](int kt, int buf) {
        const int k0 = kt * BK;
        char* dA = sA + buf * BM * 128 + uw * 1024;
        char* dW = sW + buf * BN * 128 + uw * 1024;
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) lds_load16(a_src[j] + k0, dA + j * 4096);
#pragma unroll
        for (int j = 0; j < W_LOADS; ++j) lds_load16(wv_ptr(g.W, w_src[j] + (uint64_t)k0 * 2), dW + j * 4096);
    };

    const int KT = g.K / BK;
    issue_slab(0, 0);
    __syncthreads();                     // (the compiler waits for the LDS-DMA before the barrier)

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) issue_slab(kt + 1, buf ^ 1);
        const char* cA = sA + buf * BM * 128;
        const char* cW = sW + buf * BN * 128;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 fa[MT], fw[NT];
            const int c = kk * 2 + lg;
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                const int row = wm0 + j * 32 + li;
                fa[j] = *(const bf16x8*)(cA + row * 128 + ((c ^ swz(row)) << 4));
            }
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                const int row = wn0 + i * 32 + li;
                fw[i] = *(const bf16x8*)(cW + row * 128 + ((c ^ swz(row)) << 4));
            }
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();                 // slab kt+1 has landed and slab kt is free to overwrite
    }

    // ---- epilogue: lane = token row li, register quad = 4 consecutive features
#pragma unroll
    for (int i = 0; i < NT; ++i) {
#pragma unroll
        for (int vb = 0; vb < 4; ++vb) {
            const int n = n0 + wn0 + i * 32 + vb * 8 + lg * 4;
            if (n >= g.n1) continue;                 // N and panel ends are multiples of 8
            float b[4] = {0.f, 0.f, 0.f, 0.f};
            if (g.has_bias) {
                const uint2 bb = *(const uint2*)wv_ptr(g.W, g.bias_off + 2ull * n);
                b[0] = __uint_as_float(bb.x << 16);
                b[1] = __uint_as_float(bb.x & 0xffff0000u);
                b[2] = __uint_as_float(bb.y << 16);
                b[3] = __uint_as_float(bb.y & 0xffff0000u);
            }
            float gt[4] = {1.f, 1.f, 1.f, 1.f};
            if (EPI == EPI_GATE_RESID && g.gate) {
                const float4 t = *(const float4*)(g.gate + n);
                gt[0] = t.x; gt[1] = t.y; gt[2] = t.z; gt[3] = t.w;
            }
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                const int m = m0 + wm0 + j * 32 + li;
                if (m >= g.M) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][vb * 4 + e] + b[e];
                if (EPI == EPI_SPLIT_GELU) {
                    bf16* dst;
                    if (n < g.n_split) {
                        dst = g.out0 + (size_t)m * g.ld0 + n;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = gelu_tanh_f32(v[e]);
                        dst = g.out1 + (size_t)m * g.ld1 + g.col1_off + (n - g.n_split);
                    }
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
                    *(bf16x4*)dst = o;
                } else {
                    const float4 r = *(const float4*)(g.resid + (size_t)m * g.ldy + n);
                    float4 o;
                    o.x = r.x + gt[0] * v[0];
                    o.y = r.y + gt[1] * v[1];
                    o.z = r.z + gt[2] * v[2];
                    o.w = r.w + gt[3] * v[3];
                    *(float4*)(g.y + (size_t)m * g.ldy + n) = o;
                }
            }
        }
    }
}

template <int BM, int BN, int EPI>
hipError_t launch(const GemmArgs& g, hipStream_t s) {
    const int tiles_m = (g.M + BM - 1) / BM;
    const int tiles_n = (g.n1 - g.n0 + BN - 1) / BN;
    const size_t smem = 2 * (BM + BN) * 128;
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

}  // namespace

const char* gemm_check(const GemmArgs& g) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return "gemm: empty shape";
    if (g.K % BK) return "gemm: K must be a multiple of 64";
    if (g.N % 8) return "gemm: N must be a multiple of 8";
    if (g.n0 < 0 || g.n1 > g.N || g.n0 >= g.n1 || (g.n0 % 8) || (g.n1 % 8)) return "gemm: bad feature panel";
    if (g.lda < g.K || (g.lda % 8)) return "gemm: lda must be >= K and a multiple of 8";
    if ((g.w_off % 16) || (g.has_bias && (g.bias_off % 16))) return "gemm: weight/bias offsets must be 16-byte aligned";
    if (((uintptr_t)g.A) % 16) return "gemm: A must be 16-byte aligned";
    if (g.epi == EPI_SPLIT_GELU) {
        if (g.n_split % 8) return "gemm: n_split must be a multiple of 8";
        if (g.n_split > 0 && (!g.out0 || (g.ld0 % 4) || ((uintptr_t)g.out0 % 8))) return "gemm: bad out0";
        if (g.n_split < g.N && (!g.out1 || (g.ld1 % 4) || (g.col1_off % 4) || ((uintptr_t)g.out1 % 8))) return "gemm: bad out1";
    } else if (g.epi == EPI_GATE_RESID) {
        if (!g.resid || !g.y || (g.ldy % 4) || ((uintptr_t)g.y % 16) || ((uintptr_t)g.resid % 16)) return "gemm: bad residual/output";
        if (g.gate && ((uintptr_t)g.gate % 16)) return "gemm: gate must be 16-byte aligned";
    } else {
        return "gemm: unknown epilogue";
    }
    return nullptr;
}

int gemm_tile(const GemmArgs& g) {
    // Small problems take 128x128 tiles so that the grid still covers the chip.
    const long tiles256 = (long)((g.M + 255) / 256) * ((g.n1 - g.n0 + 255) / 256);
    return tiles256 >= 128 ? 256 : 128;
}

hipError_t gemm_launch(const GemmArgs& g, hipStream_t s) {
    const bool big = gemm_tile(g) == 256;
    if (g.epi == EPI_SPLIT_GELU)
        return big ? launch<256, 256, EPI_SPLIT_GELU>(g, s) : launch<128, 128, EPI_SPLIT_GELU>(g, s);
    return big ? launch<256, 256, EPI_GATE_RESID>(g, s) : launch<128, 128, EPI_GATE_RESID>(g, s);
}
