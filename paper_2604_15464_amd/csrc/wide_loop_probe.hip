// Measurement program, not part of the library: the instruction stream of the
// wide kernel's loop over one 64-position K/V tile (32 rows per wave, head_dim
// 128, bf16; Alg. 1 inner step: S = Q K^T, online softmax, O += P V) with its
// operands in LDS and no global memory traffic, timed in wall time (HIP events)
// and with the shader's own counter (s_memtime).  It answers two questions
// about the bound of the wide kernel on this chip:
//   - what fraction of the nominal MFMA rate (32 cycles per 32x32x16 bf16 MFMA
//     at 2.4 GHz) a loop of MFMAs alone, and the attention loop in different
//     orders of the same work (the kernel's order with one barrier per tile; the
//     same without a barrier; the second wave of every SIMD one block out of
//     phase), sustain on a few CUs and on all of them;
//   - how the s_memtime counter behaves meanwhile (it slows down with the load:
//     it is no fixed-rate clock, and wall time is the figure that counts).
//
//   hipcc --offload-arch=gfx950 -O3 wide_loop_probe.hip -o wide_loop_probe
//   ./wide_loop_probe [workgroups, default 256]
//
// The LDS tile, its swizzle and the operand reads are those of rpa_wide_kernel
// (K by ds_read_b128, V by the transposing read); the data is arbitrary.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) short4v lds_short4;
typedef const __attribute__((address_space(3))) bf16x8 lds_bf16x8;

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);      \
            exit(1);                                                                   \
        }                                                                              \
    } while (0)

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    f32x2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}
__device__ __forceinline__ float max_across_halves(float x) {
    float lo = x, hi = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(lo), "+v"(hi));
    return fmaxf(lo, hi);
}

constexpr int ROWB = 256, TILEB = 64 * ROWB, STAGEB = 2 * TILEB, STAGES = 3;
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

enum Order { KERNEL_ORDER = 0, ROTATED = 1, MFMA_ONLY = 2 };

// ORDER KERNEL_ORDER: per 32-position half: scores, softmax, PV (what rpa_wide_kernel does).
// ORDER ROTATED: waves 4..7 (the second wave of every SIMD) run softmax and PV of
//   the previous half before the scores of this half, so that a barrier restarts
//   the two waves of a SIMD in opposite phases.
// ORDER MFMA_ONLY: the 32 MFMAs of a tile and nothing else.
template <int ORDER, bool BARRIER>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2)))
probe(float* out, uint64_t* ticks, int tiles, float scale_log2) {
    extern __shared__ uint4 smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n32 = lane & 31, h = lane >> 5;
    for (int i = threadIdx.x; i < STAGES * STAGEB / 16; i += blockDim.x) {
        const uint32_t w = 0x3c003c00u + ((i * 7) & 0xff);
        smem[i] = make_uint4(w, w + 1, w + 2, w + 3);
    }
    __syncthreads();
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)smem;
    uint32_t koff[8], voff[4][2];
    for (int kk = 0; kk < 8; ++kk) {
        koff[kk] = lds_base + n32 * ROWB + (((2 * kk + h) ^ swz(n32)) * 16);
        asm volatile("" : "+v"(koff[kk]));
    }
    {
        const int j16 = lane & 15, half16 = (lane >> 4) & 1;
        for (int jb = 0; jb < 4; ++jb)
            for (int rd = 0; rd < 2; ++rd) {
                const int r = 4 * h + (j16 >> 2) + 8 * rd;
                const int chunk = 4 * jb + 2 * half16 + ((j16 & 3) >> 1);
                voff[jb][rd] = lds_base + r * ROWB + ((chunk ^ swz(r)) * 16) + (j16 & 1) * 8;
                asm volatile("" : "+v"(voff[jb][rd]));
            }
    }
    bf16x8 qreg[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        union {
            uint32_t w[4];
            bf16x8 v;
        } q;
#pragma unroll
        for (int e = 0; e < 4; ++e) q.w[e] = pack_bf16(0.01f * (lane + kk + 2 * e), 0.01f * (lane + kk + 2 * e + 1));
        qreg[kk] = q.v;
    }
    f32x16 o[4];
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) o[j][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const uint64_t t_begin = __builtin_amdgcn_s_memtime();
    union VOp {
        short4v p[2];
        bf16x8 v;
    };

    auto scores = [&](uint32_t ldsK) __attribute__((always_inline)) -> f32x16 {
        f32x16 s;
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
        bf16x8 kop[8];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) kop[kk] = (bf16x8) * (lds_bf16x8*)(uintptr_t)(koff[kk] + ldsK);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kk], qreg[kk], s, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        return s;
    };
    auto softmax_pv = [&](f32x16 s, uint32_t ldsV) __attribute__((always_inline)) {
        VOp vop[2][4];
#pragma unroll
        for (int jb = 0; jb < 4; ++jb)
#pragma unroll
            for (int rd = 0; rd < 2; ++rd)
                vop[0][jb].p[rd] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(uintptr_t)(voff[jb][rd] + ldsV));
        __builtin_amdgcn_sched_barrier(0);
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[v]);
        mx = max_across_halves(mx) * scale_log2;
        const float m_new = (mx > m_run + 8.f) ? mx : m_run; // thresholded reference maximum
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[v], scale_log2, -m_use));
            s[v] = pv;
            psum += pv;
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] *= alpha;
        }
        bf16x8 pop[2];
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            union {
                uint32_t w[4];
                bf16x8 v;
            } pk;
#pragma unroll
            for (int e = 0; e < 4; ++e) pk.w[e] = pack_bf16(s[8 * kh + 2 * e], s[8 * kh + 2 * e + 1]);
            pop[kh] = pk.v;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int jb = 0; jb < 4; ++jb)
#pragma unroll
            for (int rd = 0; rd < 2; ++rd)
                vop[1][jb].p[rd] =
                    __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(uintptr_t)(voff[jb][rd] + ldsV + 16 * ROWB));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int jb = 0; jb < 4; ++jb)
                o[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[kh][jb].v, pop[kh], o[jb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    };

    if constexpr (ORDER == MFMA_ONLY) {
        // operands rotate over four register sets each (one fixed A operand for every
        // MFMA runs 15 % slower)
        for (int t = 0; t < tiles; ++t) {
#pragma unroll
            for (int i = 0; i < 32; ++i)
                o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qreg[i & 3], qreg[4 + ((i >> 2) & 3)], o[i & 3], 0, 0, 0);
            if (BARRIER) __syncthreads();
        }
    } else if (ORDER == KERNEL_ORDER || wave < 4) {
        for (int t = 0; t < tiles; ++t) {
            const uint32_t stage = (t % STAGES) * STAGEB;
            softmax_pv(scores(stage), stage + TILEB);
            softmax_pv(scores(stage + 32 * ROWB), stage + TILEB + 32 * ROWB);
            if (BARRIER) __syncthreads();
        }
    } else {
        f32x16 s_prev;
        for (int v = 0; v < 16; ++v) s_prev[v] = 0.f;
        uint32_t v_prev = TILEB + 32 * ROWB;
        for (int t = 0; t < tiles; ++t) {
            const uint32_t stage = (t % STAGES) * STAGEB;
            softmax_pv(s_prev, v_prev);
            softmax_pv(scores(stage), stage + TILEB);
            s_prev = scores(stage + 32 * ROWB);
            v_prev = stage + TILEB + 32 * ROWB;
            if (BARRIER) __syncthreads();
        }
    }
    float r = l_run + m_run;
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) r += o[j][v];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = r;
    const uint64_t t_end = __builtin_amdgcn_s_memtime();
    if (threadIdx.x == 0 && blockIdx.x == gridDim.x - 1) ticks[0] = t_end - t_begin;
}

template <int ORDER, bool BARRIER>
static void run(const char* name, float* out, uint64_t* ticks, int nblk) {
    const int tiles = 5994; // a multiple of the ring depth; long enough for the set-up not to count
    CK(hipFuncSetAttribute((const void*)probe<ORDER, BARRIER>, hipFuncAttributeMaxDynamicSharedMemorySize,
                           STAGES * STAGEB));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    float best = 1e9f;
    uint64_t best_ticks = 0;
    for (int rep = 0; rep < 4; ++rep) {
        CK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL((probe<ORDER, BARRIER>), dim3(nblk), dim3(512), STAGES * STAGEB, 0, out, ticks, tiles, 0.1275f);
        CK(hipEventRecord(e1, 0));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        if (rep > 0 && ms < best) {
            best = ms;
            CK(hipMemcpy(&best_ticks, ticks, 8, hipMemcpyDeviceToHost));
        }
    }
    const double ticks_per_tile = (double)best_ticks / tiles;
    const double us_per_tile = best * 1e3 / tiles;
    const double mfma_nominal_us = 2048.0 / 2400.0; // 2 waves x 32 MFMAs x 32 cycles at 2.4 GHz
    printf("%-46s wg %3d: %6.3f us/tile = %4.1f %% of the nominal bf16 MFMA rate | s_memtime %6.0f ticks/tile, %4.2f per ns\n",
           name, nblk, us_per_tile, 100.0 * mfma_nominal_us / us_per_tile, ticks_per_tile, ticks_per_tile / us_per_tile * 1e-3);
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
}

int main(int argc, char** argv) {
    const int nblk = argc > 1 ? atoi(argv[1]) : 256;
    float* out;
    uint64_t* ticks;
    CK(hipMalloc(&out, (size_t)nblk * 512 * sizeof(float)));
    CK(hipMalloc(&ticks, 64));
    run<KERNEL_ORDER, true>("(warm-up)", out, ticks, nblk);
    run<MFMA_ONLY, false>("32 MFMAs per tile and nothing else", out, ticks, nblk);
    run<KERNEL_ORDER, true>("kernel's order, barrier per tile", out, ticks, nblk);
    run<KERNEL_ORDER, false>("kernel's order, no barrier", out, ticks, nblk);
    run<ROTATED, true>("second wave of a SIMD out of phase, barrier", out, ticks, nblk);
    run<ROTATED, false>("second wave of a SIMD out of phase, no barrier", out, ticks, nblk);
    run<KERNEL_ORDER, true>("kernel's order, barrier per tile (again)", out, ticks, nblk);
    CK(hipFree(out));
    CK(hipFree(ticks));
    return 0;
}
