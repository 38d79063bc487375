// Ceiling probe for the wide attention loop on gfx950 (measurement aid, not part of the library).
//
// What does the instruction mix of the prefill-tile loop reach on this device when everything that is
// specific to the real kernel (paged addressing, masks, ragged tiles, work-list scheduling) is taken away?
// Four kernels, all with 8 waves x 32 query rows per workgroup and one workgroup per CU:
//   mfma_only   back-to-back v_mfma_f32_32x32x16_bf16 on register operands: the matrix peak and the clock;
//   coexec      waves 0-3 (one per SIMD) run products only, waves 4-7 the vector work of the softmax only, each
//               group alone and both together: how much of the vector work hides under the other wave's products;
//   attn_loop   per 64 keys and wave: S^T = K Q^T (16 products, K fragments read from LDS), row max, 32 x
//               (fma, exp2, add, convert), O^T += V^T P^T (16 products, V fragments by transposing LDS reads),
//               one workgroup barrier per 128 keys -- with or without the direct global -> LDS loads of the next
//               128-key stage (64 KB per workgroup, from a buffer that stays in L2 or from one that does not);
//   attn_pipe   the same work as an in-wave software pipeline over 32-key blocks (per step one product of block
//               b+1's S^T, the exponentials of a slice of block b, one product of O^T for block b-1; fragment reads
//               three steps ahead, a scheduling fence per step), softmax without a block maximum on the common path
//               (fma, exp2, half a convert, half a bf16 dot product per logit), filled and drained inside every
//               128-key stage or running across the stage barrier.
// Every address is in bounds by construction, every loop has a fixed trip count, nothing is checked
// numerically: only the time matters.  Prints one JSON line.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <type_traits>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
#define LDS_PTR(T, a) ((__attribute__((address_space(3))) T*)(uintptr_t)(a))

__device__ unsigned long long g_clk[2];          // shader cycles and 100 MHz ticks of workgroup 0, wave 0

__global__ __launch_bounds__(512, 1) void mfma_only(float* out, int iters) {
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.25f * (float)((threadIdx.x + i) & 3));
        b[i] = (__bf16)(0.5f + 0.125f * (float)(i & 1));
    }
    f32x16 acc[2] = {f32x16{0}, f32x16{0}};
    const uint64_t c0 = __builtin_readcyclecounter(), w0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[1], 0, 0, 0);
        }
    }
    const uint64_t c1 = __builtin_readcyclecounter(), w1 = __builtin_amdgcn_s_memrealtime();
    float s = 0;
    for (int i = 0; i < 16; ++i) s += acc[0][i] + acc[1][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        g_clk[0] = c1 - c0;
        g_clk[1] = w1 - w0;
    }
}

// WHO: 1 = waves 0-3 issue 32 products per iteration, 2 = waves 4-7 do the vector work of one 64-key unit per
// iteration (32 logits: max, fma, exp2, add, convert), 3 = both at once.  The groups share no data.
template <int WHO>
__global__ __launch_bounds__(512, 1) void coexec(float* out, int iters, float c) {
    const int wave = threadIdx.x >> 6;
    float s = 0;
    if ((WHO & 1) && wave < 4) {
        bf16x8 a, b;
        for (int i = 0; i < 8; ++i) {
            a[i] = (__bf16)(0.25f * (float)((threadIdx.x + i) & 3));
            b[i] = (__bf16)(0.5f + 0.125f * (float)(i & 1));
        }
        f32x16 acc0 = f32x16{0}, acc1 = f32x16{0};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc1, 0, 0, 0);
            }
        }
        for (int i = 0; i < 16; ++i) s += acc0[i] + acc1[i];
    } else if ((WHO & 2) && wave >= 4) {
        float S[32];
        for (int i = 0; i < 32; ++i) S[i] = 0.001f * (float)(threadIdx.x + 3 * i);
        float m = 0.f, l = 0.f;
        uint32_t P[16];
        for (int it = 0; it < iters; ++it) {
            float mx = S[0];
#pragma unroll
            for (int i = 1; i < 32; ++i) mx = fmaxf(mx, S[i]);
            m = fmaxf(m, mx * c);
#pragma unroll
            for (int i = 0; i < 32; i += 2) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[i], c, -m));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[i + 1], c, -m));
                l += p0 + p1;
                typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                const bf16x2 q = {(__bf16)p0, (__bf16)p1};
                P[i / 2] = __builtin_bit_cast(uint32_t, q);
            }
#pragma unroll
            for (int i = 0; i < 32; ++i) S[i] += (float)(P[i & 15] & 0xff) * 1e-6f + l * 1e-9f;   // the next unit depends on this one
        }
        s = l + m + S[5];
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__device__ __forceinline__ void direct_load16(const char* gbase, uint32_t voff, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(gbase) : "memory");
}

// LOADS: 0 none, 1 the next stage's 64 KB by direct loads (8 per wave), issued at the start of the stage.
// src: per-workgroup region of `span` bytes (a power of two >= 64 KB), walked stage by stage.
template <int LOADS>
__global__ __launch_bounds__(512, 1) void attn_loop(float* out, const char* src, uint32_t span, int stages, float c) {
    extern __shared__ __attribute__((aligned(16))) char smem_dyn[];
    const uint32_t smem = (uint32_t)(uintptr_t)LDS_PTR(char, smem_dyn);
    for (int i = threadIdx.x; i < 32768; i += 512) ((uint32_t*)smem_dyn)[i] = 0x3c003c00u + (uint32_t)(i & 7);
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    bf16x8 Q[8];
    for (int k = 0; k < 8; ++k)
        for (int i = 0; i < 8; ++i) Q[k][i] = (__bf16)(0.01f * (float)((lane + k + i) & 7));
    f32x16 O[4] = {f32x16{0}, f32x16{0}, f32x16{0}, f32x16{0}};
    float m = 0.f, l = 0.f;
    const char* wg_src = src + (size_t)blockIdx.x * span;
    const uint64_t c0 = __builtin_readcyclecounter(), w0 = __builtin_amdgcn_s_memrealtime();
    for (int t = 0; t < stages; ++t) {
        // stage = 128 keys: K at +0 (2 units x 16 KB), V at +32 KB; two stages of 64 KB
        const uint32_t cur = smem + (t & 1) * 65536, nxt = smem + ((t + 1) & 1) * 65536;
        if (LOADS) {
            const uint32_t goff = __builtin_amdgcn_readfirstlane(((uint32_t)(t + 1) * 65536u) & (span - 1));
            const char* gsrc = wg_src + goff + wv * 8192;           // this wave's 8 KB of the next stage
#pragma unroll
            for (int g = 0; g < 8; ++g)
                direct_load16(gsrc + g * 1024, lane * 16, __builtin_amdgcn_readfirstlane(nxt + wv * 8192 + g * 1024));
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t base = cur + u * 16384;
            f32x16 S[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                S[h] = f32x16{0};
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    const bf16x8 a = __builtin_bit_cast(bf16x8, *LDS_PTR(const u32x4, base + h * 8192 + kk * 1024 + lane * 16));
                    S[h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, Q[kk], S[h], 0, 0, 0);
                }
            }
            float mx = S[0][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fmaxf(mx, S[0][i]);
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[1][i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            m = fmaxf(m, mx * c);
            bf16x8 P[2][2];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(S[h][i], c, -m));
                    l += pv;
                    P[h][i >> 3][i & 7] = (__bf16)pv;
                }
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        const uint32_t a0 = base + 32768 + h * 8192 + cc * 4096 + db * 1024 + lane * 8;
                        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0));
                        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0 + 512));
                        const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                        O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), P[h][cc], O[db], 0, 0, 0);
                    }
        }
        if (LOADS) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
    const uint64_t c1 = __builtin_readcyclecounter(), w1 = __builtin_amdgcn_s_memrealtime();
    float s = l + m;
    for (int k = 0; k < 4; ++k)
        for (int i = 0; i < 16; ++i) s += O[k][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        g_clk[0] = c1 - c0;
        g_clk[1] = w1 - w0;
    }
}

// VPLAIN: 1 = the V fragments are plain 16-byte LDS reads like the K fragments (what a d-major V tile would allow)
// instead of pairs of transposing 8-byte reads.
// ACROSS: 0 = six iterations per stage (fill, four blocks, drain), 1 = four full iterations per stage (the pipeline
// state is carried over the barrier; the V rows that an iteration uses then belong to keys 64 earlier than its K rows).
template <int ACROSS, int LOADS, int VPLAIN = 0>
__global__ __launch_bounds__(512, 1) void attn_pipe(float* out, const char* src, uint32_t span, int stages, float c) {
    extern __shared__ __attribute__((aligned(16))) char smem_dyn[];
    const uint32_t smem = (uint32_t)(uintptr_t)LDS_PTR(char, smem_dyn);
    for (int i = threadIdx.x; i < 32768; i += 512) ((uint32_t*)smem_dyn)[i] = 0x3c003c00u + (uint32_t)(i & 7);
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    bf16x8 Q[8];
    for (int k = 0; k < 8; ++k)
        for (int i = 0; i < 8; ++i) Q[k][i] = (__bf16)(0.01f * (float)((lane + k + i) & 7));
    f32x16 O[4] = {f32x16{0}, f32x16{0}, f32x16{0}, f32x16{0}};
    float m = 0.f, l = 0.f;
    f32x16 Sa = f32x16{0}, Sb = f32x16{0};
    bf16x8 Pa[2], Pb[2];
    for (int i = 0; i < 8; ++i) Pa[0][i] = Pa[1][i] = Pb[0][i] = Pb[1][i] = (__bf16)0.01f;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    constexpr int PF = 3;
    // S_nxt <- K block at kq; P_cur <- exponentials of S_cur; O += V block at vp times P_prev
    auto iter = [&](uint32_t kq, uint32_t vp, auto has_qk, auto has_sm, auto has_pv, f32x16& S_cur, f32x16& S_nxt,
                    bf16x8 (&P_cur)[2], bf16x8 (&P_prev)[2]) {
        constexpr bool QK = decltype(has_qk)::value, SM = decltype(has_sm)::value, PV = decltype(has_pv)::value;
        auto rdk = [&](int j) { return __builtin_bit_cast(bf16x8, *LDS_PTR(const u32x4, kq + j * 1024 + lane * 16)); };
        auto rdv = [&](int j) {
            if (VPLAIN) return __builtin_bit_cast(bf16x8, *LDS_PTR(const u32x4, vp + j * 1024 + lane * 16));
            const uint32_t a0 = vp + (j / 4) * 4096 + (j % 4) * 1024 + lane * 8;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0 + 512));
            const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            return __builtin_bit_cast(bf16x8, av);
        };
        bf16x8 kf[8], vf[8];
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            if (QK) kf[j] = rdk(j);
            if (PV) vf[j] = rdv(j);
        }
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j + PF < 8) {
                if (QK) kf[j + PF] = rdk(j + PF);
                if (PV) vf[j + PF] = rdv(j + PF);
            }
            if (QK) S_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], Q[j], j == 0 ? f32x16{0} : S_nxt, 0, 0, 0);
            if (SM) {
                const bf16x2 pr = {(__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(S_cur[2 * j], c, -m)),
                                   (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(S_cur[2 * j + 1], c, -m))};
                psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
                P_cur[(2 * j) >> 3][(2 * j) & 7] = pr[0];
                P_cur[(2 * j) >> 3][(2 * j + 1) & 7] = pr[1];
            }
            if (PV) O[j % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[j], P_prev[j / 4], O[j % 4], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (SM) {
            if (__any(!(psum <= 4096.0f))) {            // the rare path of the real kernel; never taken here
                m += 12.0f;
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int i = 0; i < 16; ++i) O[k][i] *= 0.000244140625f;
                l *= 0.000244140625f;
            }
            l += psum;
        }
    };
    using T = std::true_type;
    using F = std::false_type;
    const char* wg_src = src + (size_t)blockIdx.x * span;
    const uint64_t c0 = __builtin_readcyclecounter(), w0 = __builtin_amdgcn_s_memrealtime();
    for (int t = 0; t < stages; ++t) {
        const uint32_t cur = smem + (t & 1) * 65536, nxt = smem + ((t + 1) & 1) * 65536;
        if (LOADS) {
            const uint32_t goff = __builtin_amdgcn_readfirstlane(((uint32_t)(t + 1) * 65536u) & (span - 1));
            const char* gsrc = wg_src + goff + wv * 8192;
#pragma unroll
            for (int g = 0; g < 8; ++g)
                direct_load16(gsrc + g * 1024, lane * 16, __builtin_amdgcn_readfirstlane(nxt + wv * 8192 + g * 1024));
        }
        auto kb = [&](int b) { return cur + (b >> 1) * 16384 + (b & 1) * 8192; };      // K rows of block b
        auto vb = [&](int b) { return kb(b) + 32768; };                                // V rows of block b
        if (ACROSS) {
            iter(kb(0), vb(0), T{}, T{}, T{}, Sb, Sa, Pb, Pa);
            iter(kb(1), vb(1), T{}, T{}, T{}, Sa, Sb, Pa, Pb);
            iter(kb(2), vb(2), T{}, T{}, T{}, Sb, Sa, Pb, Pa);
            iter(kb(3), vb(3), T{}, T{}, T{}, Sa, Sb, Pa, Pb);
        } else {
            iter(kb(0), 0, T{}, F{}, F{}, Sb, Sa, Pb, Pa);
            iter(kb(1), 0, T{}, T{}, F{}, Sa, Sb, Pa, Pb);
            iter(kb(2), vb(0), T{}, T{}, T{}, Sb, Sa, Pb, Pa);
            iter(kb(3), vb(1), T{}, T{}, T{}, Sa, Sb, Pa, Pb);
            iter(0, vb(2), F{}, T{}, T{}, Sb, Sa, Pb, Pa);
            iter(0, vb(3), F{}, F{}, T{}, Sa, Sb, Pa, Pb);
        }
        if (LOADS) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
    const uint64_t c1 = __builtin_readcyclecounter(), w1 = __builtin_amdgcn_s_memrealtime();
    float s = l + m;
    for (int k = 0; k < 4; ++k)
        for (int i = 0; i < 16; ++i) s += O[k][i] + (k == 0 ? Sa[i] + Sb[i] : 0.f);
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        g_clk[0] = c1 - c0;
        g_clk[1] = w1 - w0;
    }
}

#define CK(x)                                                                        \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            fprintf(stderr, "%s: %s (line %d)\n", #x, hipGetErrorString(e_), __LINE__); \
            return 1;                                                                \
        }                                                                            \
    } while (0)

struct Result {
    double ms, ghz;
};

template <class F>
static int measure(F&& launch, int warm, int reps, Result* r) {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    for (int i = 0; i < warm; ++i) launch();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int i = 0; i < reps; ++i) launch();
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms = 0;
    CK(hipEventElapsedTime(&ms, e0, e1));
    unsigned long long clk[2];
    CK(hipMemcpyFromSymbol(clk, HIP_SYMBOL(g_clk), sizeof(clk)));
    r->ms = ms / reps;
    r->ghz = clk[1] ? (double)clk[0] / (double)clk[1] * 0.1 : 0.0;
    CK(hipGetLastError());
    return 0;
}

int main() {
    const int NWG = 512;                               // two workgroups per CU, one after the other
    const int STAGES = 1000;                           // 128-key stages per workgroup
    float* out;
    char* src;
    const size_t span_big = 4u << 20;                  // 4 MB per workgroup: 2 GB in total, streams from HBM
    CK(hipMalloc(&out, (size_t)NWG * 512 * sizeof(float)));
    CK(hipMalloc(&src, (size_t)NWG * span_big));
    CK(hipMemset(src, 0x3c, (size_t)NWG * span_big));
    CK(hipFuncSetAttribute((const void*)attn_loop<0>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    CK(hipFuncSetAttribute((const void*)attn_loop<1>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));

    // 64 products of 32x32x16 per wave and stage, 8 waves
    const double flop_stage = 8.0 * 64.0 * 32768.0;
    Result r_mfma, r_loop, r_l2, r_hbm;
    const int MF_ITERS = 4000;                         // x 16 products
    if (measure([&] { hipLaunchKernelGGL(mfma_only, dim3(NWG), dim3(512), 0, 0, out, MF_ITERS); }, 20, 20, &r_mfma)) return 1;
    if (measure([&] { hipLaunchKernelGGL(attn_loop<0>, dim3(NWG), dim3(512), 131072, 0, out, src, 1u << 17, STAGES, 0.1f); }, 20, 20, &r_loop)) return 1;
    if (measure([&] { hipLaunchKernelGGL(attn_loop<1>, dim3(NWG), dim3(512), 131072, 0, out, src, 1u << 17, STAGES, 0.1f); }, 20, 20, &r_l2)) return 1;
    if (measure([&] { hipLaunchKernelGGL(attn_loop<1>, dim3(NWG), dim3(512), 131072, 0, out, src, (uint32_t)span_big, STAGES, 0.1f); }, 20, 20, &r_hbm)) return 1;
    Result r_p0, r_p1, r_p0l2, r_p0hbm, r_pv, r_pvl2;
    CK(hipFuncSetAttribute((const void*)attn_pipe<0, 0, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    CK(hipFuncSetAttribute((const void*)attn_pipe<0, 1, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    if (measure([&] { hipLaunchKernelGGL((attn_pipe<0, 0, 1>), dim3(NWG), dim3(512), 131072, 0, out, src, 1u << 17, STAGES, 0.1f); }, 20, 20, &r_pv)) return 1;
    if (measure([&] { hipLaunchKernelGGL((attn_pipe<0, 1, 1>), dim3(NWG), dim3(512), 131072, 0, out, src, 1u << 17, STAGES, 0.1f); }, 20, 20, &r_pvl2)) return 1;
    CK(hipFuncSetAttribute((const void*)attn_pipe<0, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    CK(hipFuncSetAttribute((const void*)attn_pipe<1, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    CK(hipFuncSetAttribute((const void*)attn_pipe<0, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    if (measure([&] { hipLaunchKernelGGL((attn_pipe<0, 0>), dim3(NWG), dim3(512), 131072, 0, out, src, 1u << 17, STAGES, 0.1f); }, 20, 20, &r_p0)) return 1;
    if (measure([&] { hipLaunchKernelGGL((attn_pipe<1, 0>), dim3(NWG), dim3(512), 131072, 0, out, src, 1u << 17, STAGES, 0.1f); }, 20, 20, &r_p1)) return 1;
    if (measure([&] { hipLaunchKernelGGL((attn_pipe<0, 1>), dim3(NWG), dim3(512), 131072, 0, out, src, 1u << 17, STAGES, 0.1f); }, 20, 20, &r_p0l2)) return 1;
    if (measure([&] { hipLaunchKernelGGL((attn_pipe<0, 1>), dim3(NWG), dim3(512), 131072, 0, out, src, (uint32_t)span_big, STAGES, 0.1f); }, 20, 20, &r_p0hbm)) return 1;
    Result r_cm, r_cv, r_cb;
    const int CO_ITERS = 2000;
    if (measure([&] { hipLaunchKernelGGL(coexec<1>, dim3(NWG), dim3(512), 0, 0, out, CO_ITERS, 0.1f); }, 5, 10, &r_cm)) return 1;
    if (measure([&] { hipLaunchKernelGGL(coexec<2>, dim3(NWG), dim3(512), 0, 0, out, CO_ITERS, 0.1f); }, 5, 10, &r_cv)) return 1;
    if (measure([&] { hipLaunchKernelGGL(coexec<3>, dim3(NWG), dim3(512), 0, 0, out, CO_ITERS, 0.1f); }, 5, 10, &r_cb)) return 1;
    const double tf_mfma = (double)NWG * 8 * MF_ITERS * 16 * 32768.0 / (r_mfma.ms * 1e-3) / 1e12;
    auto tf = [&](const Result& r) { return (double)NWG * STAGES * flop_stage / (r.ms * 1e-3) / 1e12; };
    auto tbs = [&](const Result& r) { return (double)NWG * STAGES * 65536.0 / (r.ms * 1e-3) / 1e12; };
    printf("{\"coexec_ms\": {\"products_alone\": %.3f, \"vector_work_alone\": %.3f, \"both\": %.3f}, ", r_cm.ms, r_cv.ms, r_cb.ms);
    printf("\"mfma_only\": {\"TFLOPs\": %.1f, \"shader_GHz\": %.3f}, "
           "\"attn_loop_no_loads\": {\"TFLOPs\": %.1f, \"shader_GHz\": %.3f}, "
           "\"attn_loop_direct_loads_L2\": {\"TFLOPs\": %.1f, \"shader_GHz\": %.3f, \"load_TBps\": %.2f}, "
           "\"attn_loop_direct_loads_HBM\": {\"TFLOPs\": %.1f, \"shader_GHz\": %.3f, \"load_TBps\": %.2f}, ",
           tf_mfma, r_mfma.ghz, tf(r_loop), r_loop.ghz, tf(r_l2), r_l2.ghz, tbs(r_l2), tf(r_hbm), r_hbm.ghz, tbs(r_hbm));
    printf("\"attn_pipe_no_loads\": {\"TFLOPs\": %.1f, \"shader_GHz\": %.3f}, "
           "\"attn_pipe_across_barrier_no_loads\": {\"TFLOPs\": %.1f, \"shader_GHz\": %.3f}, "
           "\"attn_pipe_direct_loads_L2\": {\"TFLOPs\": %.1f, \"shader_GHz\": %.3f}, "
           "\"attn_pipe_direct_loads_HBM\": {\"TFLOPs\": %.1f, \"shader_GHz\": %.3f}, "
           "\"attn_pipe_plain_v_reads_no_loads\": {\"TFLOPs\": %.1f, \"shader_GHz\": %.3f}, "
           "\"attn_pipe_plain_v_reads_direct_loads_L2\": {\"TFLOPs\": %.1f, \"shader_GHz\": %.3f}}\n",
           tf(r_p0), r_p0.ghz, tf(r_p1), r_p1.ghz, tf(r_p0l2), r_p0l2.ghz, tf(r_p0hbm), r_p0hbm.ghz, tf(r_pv), r_pv.ghz,
           tf(r_pvl2), r_pvl2.ghz);
    return 0;
}
