// HIP kernels for gfx950 (CDNA4, wave64): paged KV append, attention over paged K/V
// (wide = prefill tiles, narrow = decode-style split-KV items, fused in one launch) and the
// split-KV combine.
//
// Operation (paper Section 3: prefill with history l_hist = C and incremental length
// l_incr = L; decode = one token per request): query i of a row sits at position C + i
// and attends keys 0..C+i; query head hq reads KV head hq / G.
//
// Matrix-core formulation.  Everything is computed transposed so that all softmax state is
// per lane:
//   S^T[key][q]  = K[key][:] . Q[q][:]          v_mfma_f32_32x32x16_bf16, A = K rows, B = Q^T
//   O^T[d][q]   += V^T[d][key] . P^T[key][q]    A = V^T (LDS transpose read), B = P^T
// In the 32x32 accumulator layout lane l owns column q = l % 32 and rows
// (i/4)*8 + (l/32)*4 + i%4 for register i, so a lane's 16 registers of S^T are 16 keys of
// ONE query row: row max / row sum are in-lane reductions plus one exchange with lane l^32,
// and the bf16 P^T operand of the second product is built from the same registers without
// leaving the register file.  The V^T operand needs 4 consecutive keys per lane for a
// fixed d; ds_read_b64_tr_b16 delivers exactly that from [key][d] data in LDS.
// Narrow items of at most 16 query rows (a decode row's grouped heads) use the same formulation on
// v_mfma_f32_16x16x32_bf16 tiles (lane l owns column q = l % 16 and keys 4 (l/16) + i, 16 + 4 (l/16) + i):
// half the matrix and softmax work per key of the 32-row tiles, most of which would be padding there.
//
// LDS tile layout ("groups"): keys are stored in groups of KPW = 64 / (d/8) keys (4 for
// d = 128), one group = exactly the 1 KB that one wave-wide 16-byte-per-lane load delivers.
// Inside a group, 64-byte quads of chunks stay together and the keys interleave:
//   addr(key, chunk) = (key / KPW) * GS + (chunk / 4) * (KPW * 64) + (key % KPW) * 64 + (chunk % 4) * 16,
//   GS = 1024 + 16.
// With this order (a) a wave's direct global->LDS load (lane i -> LDS slot i) fills a group
// while every 4 consecutive lanes fetch 64 contiguous bytes of one key row, (b) the 16 lanes
// that read one chunk of 16 consecutive keys for the first product hit 64 distinct banks
// (4 keys 64 B apart per group, groups shifted by the 16-byte pad), the 32 lanes of a
// transpose read for the second product touch 256 contiguous bytes, and (c) every operand
// address is a per-lane base plus a compile-time constant.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "kernels.h"

namespace ampd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(uintptr_t)(p))
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

constexpr int WG = 256;                 // append / combine kernels
constexpr int AWG = 64 * ATTN_WAVES;    // attention kernel: 8 waves, one workgroup per CU
constexpr int KT = 128;                 // keys per LDS stage of a wide item (one barrier per stage)
constexpr int NSTAGE = 2;               // LDS ring of K/V stages for wide items
constexpr float NEG_INF = -__builtin_inff();

template <int D>
struct Geo {
    static constexpr int CPK = D / 8;                  // 16-byte (8-element) chunks per key row
    static constexpr int KPW = 64 / CPK;               // keys per group (one wave-wide load)
    static constexpr int GS = 1024 + 16;               // LDS bytes per group
    static constexpr int B32 = (32 / KPW) * GS;        // bytes of a 32-key block (K or V)
    static constexpr int KTILE = (KT / 32) * B32;      // bytes of KT keys (K or V)
    static constexpr int WIDE_STAGE = 2 * KTILE;       // KT keys of K, then KT keys of V
    static constexpr int MERGE = ATTN_WAVES * 32 * (D + 4) * 4 + ATTN_WAVES * 32 * 2 * 4;   // narrow items: waves x (O, m, l)
    static constexpr int NARROW = ATTN_WAVES * 2 * B32;                // one private 32-key K+V block per wave
    static constexpr int SMEM0 = NSTAGE * WIDE_STAGE > MERGE ? NSTAGE * WIDE_STAGE : MERGE;
    static constexpr int SMEM = SMEM0 > NARROW ? SMEM0 : NARROW;
    static constexpr int NDB = D / 32;                 // 32-row blocks of O^T
    static constexpr int NKK = D / 16;                 // MFMA k-steps of the first product
};

// ---------------------------------------------------------------------------------------------
// small helpers

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Exchange with lane^32 folded into the reduction: v_permlane32_swap(x, x) returns
// r0 = {x[0..31], x[0..31]} and r1 = {x[32..63], x[32..63]} (by destination lane halves), so
// op(r0, r1) is op(x[l], x[l^32]) in every lane.
__device__ __forceinline__ float max_xor32(float x) {
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xor32(float x) {
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 8 stored elements -> 8 bf16 (as a 16-byte vector) for LDS.
template <int KVT>
struct RawChunk;
template <>
struct RawChunk<KV_BF16> {
    u32x4 v;
    static constexpr int ES = 2;                      // bytes per stored element
    __device__ __forceinline__ void zero() { v = u32x4{0, 0, 0, 0}; }
    __device__ __forceinline__ void load(const char* base, uint32_t lane_off) {
        v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + lane_off));   // streamed once: do not displace L2 lines
    }
    __device__ __forceinline__ u32x4 widen(float) const { return v; }
};
template <>
struct RawChunk<KV_FP8> {
    u32x4 v;                                          // 16 codes: two neighbouring chunks of one key row
    static constexpr int ES = 1;
    __device__ __forceinline__ void zero() { v = u32x4{0, 0, 0, 0}; }
    __device__ __forceinline__ void load(const char* base, uint32_t lane_off) {
        v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + lane_off));
    }
    // decode(code) * scale is exact in bf16: 4 significant bits times a power of two.  The page scales are
    // powers of two (the append kernel writes no others), so the hardware's scaled conversion, which applies
    // the exponent of `scale` only, is that product: one instruction per two elements.
    __device__ __forceinline__ static u32x4 widen8(uint32_t lo, uint32_t hi, float scale) {
        const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, scale, false);
        const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, scale, true);
        const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, scale, false);
        const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, scale, true);
        return u32x4{__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b), __builtin_bit_cast(uint32_t, c),
                     __builtin_bit_cast(uint32_t, d)};
    }
    __device__ __forceinline__ u32x4 widen_first(float scale) const { return widen8(v.x, v.y, scale); }
    __device__ __forceinline__ u32x4 widen_second(float scale) const { return widen8(v.z, v.w, scale); }
};

struct ItemCtx {
    int req, kvh, g0, gn, q0, nq, kv_begin, kv_end, part_off;
    int C, row_off;
    int c_rows;                // keys from this position on are read from the packed new rows (k_new / v_new), not from
                               // the pages: C when the page writes of this call ride in the same launch, else "never"
    const int32_t* bt_row;     // block-table row of the request
};
constexpr int NEVER = 0x3fffffff;

__device__ __forceinline__ ItemCtx load_item(const AttnParams& p, int idx) {
    const Item it = p.items[idx];
    ItemCtx c;
    c.req = it.req;
    c.kvh = it.heads & 0xff;
    c.g0 = (it.heads >> 8) & 0xff;
    c.gn = (it.heads >> 16) & 0xff;
    c.q0 = it.q0;
    c.nq = it.nq;
    c.kv_begin = it.kv_begin;
    c.kv_end = it.kv_end;
    c.part_off = it.part_off;
    c.C = it.C;
    c.row_off = it.row_off;
    c.c_rows = p.k_new ? it.C : NEVER;
    c.bt_row = p.block_table + (int64_t)it.req * p.max_pages;
    return c;
}

// Per-lane state of one wave: 32 query rows (lane % 32), O^T as D/32 accumulator blocks.
// m is a *reference* maximum in the log2 domain (scale * log2(e) folded in), not the exact
// running maximum: it is raised (and O, l rescaled) only when probabilities against it would grow too large:
// narrow items raise it when a block maximum exceeds it by more than RESCALE_SLACK (probabilities stay below
// 2^RESCALE_SLACK); wide items when a lane's 16 probabilities of a block sum to more than PSUM_LIMIT.
// (m, l, O) remain a consistent triple, which is all the final normalisation and the split-KV
// merge need.
template <int D>
struct WaveAcc {
    f32x16 O[Geo<D>::NDB];
    float m;
    float l;      // this lane's share of the running sum (lanes l and l^32 hold halves)
};
constexpr float RESCALE_SLACK = 8.0f;
constexpr float PSUM_LIMIT = 4096.0f;

// ---------------------------------------------------------------------------------------------
// the steps of one 32-key block

// S^T = K Q^T for the 32 keys whose LDS tile starts at kl.
template <int D>
__device__ __forceinline__ void qk32(uint32_t kl, const bf16x8 (&Q)[Geo<D>::NKK], f32x16& S, int lane) {
    using G_ = Geo<D>;
    const int r = lane & 31, g = lane >> 5;
    // chunk 2*kk + g of key r
    const uint32_t ka = kl + (r / G_::KPW) * G_::GS + (r % G_::KPW) * 64 + g * 16;
    S = f32x16{0};
#pragma unroll
    for (int kk = 0; kk < G_::NKK; ++kk) {
        const u32x4 raw = *LDS_PTR(const u32x4, ka + (kk >> 1) * (G_::KPW * 64) + (kk & 1) * 32);
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), Q[kk], S, 0, 0, 0);
    }
}

// rel: per lane, (last visible key of this lane's query) - (first key of the block) - 4*(lane/32)
__device__ __forceinline__ void mask32(f32x16& S, int rel) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int koff = (i >> 2) * 8 + (i & 3);
        S[i] = koff <= rel ? S[i] : NEG_INF;
    }
}

__device__ __forceinline__ float rowmax32(const f32x16& S) {
    float mx = S[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, S[i]);
    return max_xor32(mx);
}

// Raise the reference maximum to cover mx (log2 domain) and rescale O and l.
template <int D>
__device__ __forceinline__ void raise_reference(WaveAcc<D>& st, float mx) {
    const float m_new = fmaxf(st.m, mx);
    const float alpha = fast_exp2(st.m - (m_new == NEG_INF ? 0.0f : m_new));
    st.l *= alpha;
#pragma unroll
    for (int db = 0; db < Geo<D>::NDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) st.O[db][i] *= alpha;
    st.m = m_new;
}

// p = 2^(S*c - m); returns this lane's sum; P = bf16(p) as the two B operands of the second product
__device__ __forceinline__ float exp32(const f32x16& S, float c, float m_use, bf16x8 (&P)[2]) {
    float psum = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const float pv = fast_exp2(__builtin_fmaf(S[i], c, -m_use));
        psum += pv;
        P[i >> 3][i & 7] = (__bf16)pv;
    }
    return psum;
}

// The same for the wide path: the sum is taken over the ROUNDED probabilities, two per instruction
// (dot product of a bf16 pair with (1, 1) accumulated in fp32), which is also what the second product adds up.
__device__ __forceinline__ float exp32_dot(const f32x16& S, float c, float m_use, bf16x8 (&P)[2], float psum) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
        const bf16x2 pr = {(__bf16)fast_exp2(__builtin_fmaf(S[i], c, -m_use)), (__bf16)fast_exp2(__builtin_fmaf(S[i + 1], c, -m_use))};
        psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
        P[i >> 3][i & 7] = pr[0];
        P[i >> 3][(i + 1) & 7] = pr[1];
    }
    return psum;
}

// O^T += V^T P^T for the 32 keys whose LDS tile starts at vl.
// k-slot s of MFMA cc is key 16*cc + 8*(s/4) + 4*(lane/32) + s%4 of the block.
template <int D>
__device__ __forceinline__ void pv32(uint32_t vl, const bf16x8 (&P)[2], WaveAcc<D>& st, int lane) {
    using G_ = Geo<D>;
    const int g = lane >> 5, hi = (lane >> 4) & 1, i16 = lane & 15;
    // the 16 lanes of a transpose read address 4 keys (4*g + i16/4 ..) x 16 consecutive d
    const int key = 4 * g + (i16 >> 2);
    // inside the 64-byte quad of d block db: bytes hi*32 + (i16&3)*8
    const uint32_t va = vl + (key / G_::KPW) * G_::GS + (key % G_::KPW) * 64 + hi * 32 + (i16 & 3) * 8;
    constexpr int K8 = (8 / G_::KPW) * G_::GS + (8 % G_::KPW) * 64;      // +8 keys
    constexpr int K16 = (16 / G_::KPW) * G_::GS;                        // +16 keys
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
#pragma unroll
        for (int db = 0; db < G_::NDB; ++db) {
            const uint32_t a0 = va + cc * K16 + db * (G_::KPW * 64);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0));
            const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0 + K8));
            const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi4[0], hi4[1], hi4[2], hi4[3]};
            st.O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), P[cc], st.O[db], 0, 0, 0);
        }
    }
}

// One 32-key block, straight: used by narrow items (bandwidth-bound, no pipelining needed).
template <int D>
__device__ __forceinline__ void block32(uint32_t kl, uint32_t vl, const bf16x8 (&Q)[Geo<D>::NKK], WaveAcc<D>& st,
                                        float c, int rel, bool masked, int lane) {
    f32x16 S;
    bf16x8 P[2];
    qk32<D>(kl, Q, S, lane);
    if (masked) mask32(S, rel);                          // wave-uniform
    const float mx = rowmax32(S) * c;
    if (__any(mx > st.m + RESCALE_SLACK)) raise_reference<D>(st, mx);
    st.l += exp32(S, c, st.m == NEG_INF ? 0.0f : st.m, P);
    pv32<D>(vl, P, st, lane);
}

// ---------------------------------------------------------------------------------------------
// The same steps for a wave of at most 16 query rows (a decode row's grouped heads), with v_mfma_f32_16x16x32_bf16:
// half the matrix and softmax work of the 32-row steps per key.  A lane owns query column lane % 16; with g = lane / 16
// it holds S^T for keys 4 k + i and 16 + 4 k + i (i < 4; k = key_group16(g)) of the block, which are also its eight k-slots
// of the second product, so P^T is again built in registers; O^T tile dt holds d = 16 dt + 4 g + i.

__device__ __forceinline__ float max_xor16(float x) {      // as max_xor32, for lane ^ 16
    const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xor16(float x) {
    const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Which group of 4 keys (of the 16 keys of a tile) the lanes 16 g .. 16 g + 15 hold: 0, 2, 1, 3.  With this order the 32 lanes
// that one pass of a transpose read serves (g = 0, 1 or g = 2, 3) touch 256 contiguous bytes of the padded key groups
// (keys 0-3 and 8-11, or 4-7 and 12-15: LDS groups 16 bytes apart modulo 256) for d = 128; measured, the bank-conflict
// cycles of a decode launch are half of those with the order 0, 1, 2, 3.
__device__ __forceinline__ int key_group16(int g) { return ((g & 1) << 1) | ((g >> 1) & 1); }

template <int D>
struct WaveAcc16 {
    f32x4 O[D / 16];
    float m;
    float l;      // this lane's share of the running sum (the four lanes of a column hold quarters)
};

template <int D>
__device__ __forceinline__ void qk16(uint32_t kl, const bf16x8 (&Q)[D / 32], f32x4 (&S)[2], int lane) {
    using G_ = Geo<D>;
    // matrix row rho = lane % 16 carries key 4 * key_group16(rho / 4) + rho % 4 of the tile, so that lane group g ends up
    // with the keys of group key_group16(g)
    const int r = key_group16((lane & 15) >> 2) * 4 + (lane & 3), g = lane >> 4;
    // chunk 4*kk + g of key 16*t + r
    const uint32_t ka = kl + (r / G_::KPW) * G_::GS + (r % G_::KPW) * 64 + g * 16;
    constexpr int K16 = (16 / G_::KPW) * G_::GS;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        S[t] = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            const u32x4 raw = *LDS_PTR(const u32x4, ka + t * K16 + kk * (G_::KPW * 64));
            S[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, raw), Q[kk], S[t], 0, 0, 0);
        }
    }
}

// rel: per lane, (last visible key of this lane's query) - (first key of the block) - 4*key_group16(lane/16)
__device__ __forceinline__ void mask16(f32x4 (&S)[2], int rel) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) S[t][i] = 16 * t + i <= rel ? S[t][i] : NEG_INF;
}

template <int D>
__device__ __forceinline__ void raise_reference16(WaveAcc16<D>& st, float mx) {
    const float m_new = fmaxf(st.m, mx);
    const float alpha = fast_exp2(st.m - (m_new == NEG_INF ? 0.0f : m_new));
    st.l *= alpha;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) st.O[dt] *= alpha;
    st.m = m_new;
}

template <int D>
__device__ __forceinline__ void pv16(uint32_t vl, const bf16x8& P, WaveAcc16<D>& st, int lane) {
    using G_ = Geo<D>;
    const int g = lane >> 4, i16 = lane & 15;
    // the 16 lanes of a transpose read address 4 keys x 16 consecutive d and receive 4 keys of one d each
    const int key = 4 * key_group16(g) + (i16 >> 2);
    const uint32_t va = vl + (key / G_::KPW) * G_::GS + (key % G_::KPW) * 64 + (i16 & 3) * 8;
    constexpr int K16 = (16 / G_::KPW) * G_::GS;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
        const uint32_t a0 = va + (dt >> 1) * (G_::KPW * 64) + (dt & 1) * 32;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0));
        const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0 + K16));
        const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi4[0], hi4[1], hi4[2], hi4[3]};
        st.O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), P, st.O[dt], 0, 0, 0);
    }
}

template <int D>
__device__ __forceinline__ void block16(uint32_t kl, uint32_t vl, const bf16x8 (&Q)[D / 32], WaveAcc16<D>& st,
                                        float c, int rel, bool masked, int lane) {
    f32x4 S[2];
    qk16<D>(kl, Q, S, lane);
    if (masked) mask16(S, rel);                          // wave-uniform
    float mx = fmaxf(fmaxf(fmaxf(S[0][0], S[0][1]), fmaxf(S[0][2], S[0][3])), fmaxf(fmaxf(S[1][0], S[1][1]), fmaxf(S[1][2], S[1][3])));
    mx = max_xor32(max_xor16(mx)) * c;
    if (__any(mx > st.m + RESCALE_SLACK)) raise_reference16<D>(st, mx);
    const float m_use = st.m == NEG_INF ? 0.0f : st.m;
    bf16x8 P;
    float psum = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float pv = fast_exp2(__builtin_fmaf(S[i >> 2][i & 3], c, -m_use));
        psum += pv;
        P[i] = (__bf16)pv;
    }
    st.l += psum;
    pv16<D>(vl, P, st, lane);
}

// ---------------------------------------------------------------------------------------------
// Software-pipelined processing of one LDS stage by one wave, at 32-key granularity.
//
// On this device the vector instructions of the softmax hide behind matrix instructions mostly when both come
// from the SAME wave, finely interleaved in program order (a SIMD running the products of one wave and the vector
// work of another needs the products' time plus two thirds of the vector work's time; interleaved in one wave, one
// quarter).  One pipeline iteration therefore carries, step by step,
//     one product of S^T(b+1) = K(b+1) Q^T,   the exponentials of a slice of block b,   one product of O^T += V(b-1)^T P(b-1)^T
// for three consecutive 32-key blocks, with the LDS fragment reads three steps ahead; scheduling fences keep the steps
// in this order.  The pipeline is filled and drained inside every stage (6 iterations for 4 blocks), because the next
// stage's K rows are only known to have landed after the barrier that ends this one.
//
// The exponentials of a block are taken against the reference the row already has; the block's own maximum is only
// looked at when that turned out too low (some probability above 2^12: the lane's sum says so) or when the row has
// no reference yet.  That check sits at the end of the iteration, where S^T(b) is still in registers and O holds the
// blocks up to b-1: the reference is raised, O and l are rescaled, and P(b) is redone in place.

// f(integral_constant<int, I>) for I = I0 .. N-1, unrolled at compile time (a runtime loop, even one marked for
// unrolling, leaves the fragment arrays below indexed at run time, i.e. in scratch memory)
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}


template <int D>
struct PipeState {
    f32x16 S[2];            // logits of two consecutive blocks (block b lives in S[b & 1])
    bf16x8 P[2][2];         // probabilities of two consecutive blocks
};

// All blocks of one stage (NB = KT / 32 blocks; K rows at kst, V rows at vst), for one wave: NB + 2 iterations of NS
// steps, written as one flat sequence of steps so that the fragment reads also run ahead across the iterations'
// ends (only the first PF steps of a stage wait for their LDS reads).  In iteration i, block i is multiplied
// (QK, i < NB), block i-1 exponentiated (SM), block i-2 multiplied into O (PV).
//   rel0: (last visible key of the lane's row) - (first key of the stage) - 4 * (lane / 32) (read when MASK).
template <int D, bool MASK>
__device__ __forceinline__ void stage_pipelined(uint32_t kst, uint32_t vst, const bf16x8 (&Q)[Geo<D>::NKK], WaveAcc<D>& st,
                                                PipeState<D>& ps, float c, int rel0, int lane) {
    using G_ = Geo<D>;
    constexpr int NB = KT / 32;
    constexpr int NS = G_::NKK;                      // steps per iteration: one K fragment and one V fragment per step
    constexpr int LPS = 16 / NS;                     // logits per lane and step
    constexpr int PF = 3;                            // fragment reads run this many steps ahead (2 to 4 measure alike, 5 and 6 slower)
    constexpr int NSTEP = (NB + 2) * NS;
    static_assert(2 * G_::NDB == NS && LPS % 2 == 0, "steps per block");
    const int g = lane >> 5, r = lane & 31, hi = (lane >> 4) & 1, i16 = lane & 15;
    const uint32_t ka = kst + (r / G_::KPW) * G_::GS + (r % G_::KPW) * 64 + g * 16;
    const int key = 4 * g + (i16 >> 2);
    const uint32_t va = vst + (key / G_::KPW) * G_::GS + (key % G_::KPW) * 64 + hi * 32 + (i16 & 3) * 8;
    constexpr int K8 = (8 / G_::KPW) * G_::GS + (8 % G_::KPW) * 64;      // +8 keys
    constexpr int K16 = (16 / G_::KPW) * G_::GS;                        // +16 keys
    // the fragments step t needs: K fragment t % NS of block t / NS (t < NB * NS), V fragment of block t / NS - 2
    u32x4 kf[NSTEP];
    s16x8 vf[NSTEP];
    auto fetch = [&](int t) {
        const int i = t / NS, j = t % NS;
        if (i < NB) kf[t] = *LDS_PTR(const u32x4, ka + i * G_::B32 + (j >> 1) * (G_::KPW * 64) + (j & 1) * 32);
        if (i >= 2) {                                // fragment j = cc * NDB + db
            const uint32_t a0 = va + (i - 2) * G_::B32 + (j / G_::NDB) * K16 + (j % G_::NDB) * (G_::KPW * 64);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0));
            const s16x4 h4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0 + K8));
            vf[t] = s16x8{lo[0], lo[1], lo[2], lo[3], h4[0], h4[1], h4[2], h4[3]};
        }
    };
    static_for<0, PF>([&](auto tc) { fetch(decltype(tc)::value); });
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    float m_use = 0.0f, psum = 0.0f;
    static_for<0, NSTEP>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        constexpr int i = t / NS, j = t % NS;
        constexpr bool QK = i < NB, SM = i >= 1 && i <= NB, PV = i >= 2;
        f32x16& S_out = ps.S[i & 1];
        f32x16& S_in = ps.S[(i + 1) & 1];            // block i - 1
        bf16x8 (&P_out)[2] = ps.P[(i + 1) & 1];
        const bf16x8 (&P_prev)[2] = ps.P[i & 1];     // block i - 2
        if constexpr (t + PF < NSTEP) fetch(t + PF);
        if constexpr (SM && j == 0) {
            if (MASK) mask32(S_in, rel0 - 32 * (i - 1));
            m_use = st.m == NEG_INF ? 0.0f : st.m;
            psum = 0.0f;
        }
        if constexpr (QK)
            S_out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[t]), Q[j], j == 0 ? f32x16{0} : S_out, 0, 0, 0);
        // the slice's exponentials go half before and half behind the second product, so that each half runs in the
        // shadow of one matrix instruction of this wave
        float p_even[LPS / 2];
        if constexpr (SM) {
#pragma unroll
            for (int h = 0; h < LPS / 2; ++h) p_even[h] = fast_exp2(__builtin_fmaf(S_in[j * LPS + 2 * h], c, -m_use));
        }
        if constexpr (SM && PV) __builtin_amdgcn_sched_barrier(0);
        if constexpr (PV)
            st.O[j % G_::NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[t]), P_prev[j / G_::NDB],
                                                                        st.O[j % G_::NDB], 0, 0, 0);
        if constexpr (SM) {
#pragma unroll
            for (int h = 0; h < LPS / 2; ++h) {
                const int e = j * LPS + 2 * h;
                const bf16x2 pr = {(__bf16)p_even[h], (__bf16)fast_exp2(__builtin_fmaf(S_in[e + 1], c, -m_use))};
                psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
                P_out[e >> 3][e & 7] = pr[0];
                P_out[e >> 3][(e + 1) & 7] = pr[1];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (SM && j == NS - 1) {
            if (__any(st.m == NEG_INF || !(psum <= PSUM_LIMIT))) {                    // rare
                raise_reference<D>(st, rowmax32(S_in) * c);
                psum = exp32_dot(S_in, c, st.m == NEG_INF ? 0.0f : st.m, P_out, 0.0f);
            }
            st.l += psum;
        }
    });
}

// Load the B operand (Q^T) of one wave: lane holds row lane%32, d = kk*16 + (lane/32)*8 .. +8.
template <int D>
__device__ __forceinline__ void load_q(const AttnParams& p, const ItemCtx& ic, int tok, int head_in_group,
                                       bool valid, int lane, bf16x8 (&Q)[Geo<D>::NKK]) {
    const int g = lane >> 5;
    if (valid) {
        const int hq = ic.kvh * (p.Hq / p.Hkv) + ic.g0 + head_in_group;
        const char* src = static_cast<const char*>(p.q) + (((int64_t)(ic.row_off + tok) * p.Hq + hq) * D + g * 8) * 2;
#pragma unroll
        for (int kk = 0; kk < Geo<D>::NKK; ++kk)
            Q[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + kk * 32));
    } else {
#pragma unroll
        for (int kk = 0; kk < Geo<D>::NKK; ++kk) Q[kk] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
    }
}

// The same for a wave of 16 rows: lane holds row lane%16, d = kk*32 + (lane/16)*8 .. +8.
template <int D>
__device__ __forceinline__ void load_q16(const AttnParams& p, const ItemCtx& ic, int tok, int head_in_group,
                                         bool valid, int lane, bf16x8 (&Q)[D / 32]) {
    const int g = lane >> 4;
    if (valid) {
        const int hq = ic.kvh * (p.Hq / p.Hkv) + ic.g0 + head_in_group;
        const char* src = static_cast<const char*>(p.q) + (((int64_t)(ic.row_off + tok) * p.Hq + hq) * D + g * 8) * 2;
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk)
            Q[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(src + kk * 64));
    } else {
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) Q[kk] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
    }
}

// One wave-wide direct global -> LDS load: lane i moves the 16 bytes at gbase + voff_i to LDS
// byte lds + 16 i (gbase and lds wave-uniform; the LDS base travels in M0).  Written as inline
// assembly so that the compiler does not track it: its own LDS reads of the *other* pipeline
// stage would otherwise wait for these loads.  dma_wait() must precede the barrier that
// publishes the data.  Compiler-issued vmcnt waits stay correct: vector-memory loads retire in
// order, so extra loads in flight only make them stricter.  M0 is named as clobbered so that the compiler never
// assumes a value of its own survives the statement (it is a reserved register, which the compiler reports with a
// warning that is silenced here: nothing has to be preserved, M0 is rewritten before every use).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const char* gbase, uint32_t voff, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(gbase)
                 : "memory", "m0");
}
#pragma clang diagnostic pop
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---------------------------------------------------------------------------------------------
// K/V tile loader.  NTHR threads move NKEYS consecutive keys (K and V rows) from the paged
// pools into LDS, one group (KPW keys, 1 KB) per wave and pass.  Page ids are fetched one
// tile earlier than the rows they address, so that the dependent block-table -> pool load
// chain is never on the critical path; a group never straddles a page, so the page id is
// wave-uniform: it is moved to a scalar register and the 64-bit address arithmetic runs on
// the scalar unit.  Lane i fetches the chunk that belongs in LDS slot i of its group.
//   DMA = true  (bf16 cache): global -> LDS directly (global_load_lds_dwordx4), no staging
//                 registers; the data is in LDS once the vector-memory counter has drained,
//                 which the barrier that ends a pipeline step waits for.
//   DMA = false: global -> registers (fetch_kv) -> LDS (commit), widening 8-bit codes.
template <int D, int KVT, int NTHR, int NKEYS>
struct Loader {
    using G_ = Geo<D>;
    static constexpr int KPW = G_::KPW;
    static constexpr int NGRP = NKEYS / KPW;          // groups per tile
    static constexpr int NW = NTHR / 64;              // cooperating waves
    // 8-bit cache: a wave moves two consecutive groups per pass, 16 codes per lane (lanes 0-31 the first group, 32-63 the
    // second; a lane fills two neighbouring LDS slots): half as many loads and address computations per byte as with
    // one 8-byte chunk per lane.  Two groups are 8 or 16 keys from a multiple of that, so they share a page too.
    static constexpr int GPP = KVT == KV_FP8 ? 2 : 1; // groups per wave and pass
    static constexpr int KPP = GPP * KPW;             // keys per wave and pass
    static constexpr int NPASS = NGRP / (NW * GPP);
    static_assert(NPASS >= 1 && NPASS * NW * GPP == NGRP, "tile, waves and passes");
    static constexpr int ES = RawChunk<KVT>::ES;
    int pg[NPASS];
    RawChunk<KVT> k[NPASS], v[NPASS];
    // 8-bit cache: the page scales of the tile.  One per pass in general; the one-wave loader of narrow items (32 keys from a
    // multiple of 32) sees at most two pages (page size >= 16), and keeps two scales instead of eight per operand.
    static constexpr bool TWO_SCALES = NW == 1 && NKEYS == 32;
    static constexpr int NSC = TWO_SCALES ? 2 : NPASS;
    float ks[NSC], vs[NSC];
    __device__ __forceinline__ float k_scale_of(const AttnParams& p, int ps) const {
        if constexpr (TWO_SCALES) return ps * KPP < p.P ? ks[0] : ks[1];
        else return ks[ps];
    }
    __device__ __forceinline__ float v_scale_of(const AttnParams& p, int ps) const {
        if constexpr (TWO_SCALES) return ps * KPP < p.P ? vs[0] : vs[1];
        else return vs[ps];
    }

    // t: thread index inside the group of NTHR threads.  The block table is read through the
    // scalar cache (it is constant for the duration of the kernel): scalar loads do not count
    // as vector-memory loads, so waiting for a page id never waits for K/V data in flight.
    // (They do share a counter with LDS reads: the register-staged paths and the first stage
    // of a wide item use this variant, the direct-load pipeline uses fetch_pages_v below.)
    __device__ __forceinline__ void fetch_pages(const AttnParams& p, const ItemCtx& ic, int kbase, int t) {
        const auto* bt = reinterpret_cast<const __attribute__((address_space(4))) int32_t*>(
            reinterpret_cast<uintptr_t>(ic.bt_row));
        const int w = __builtin_amdgcn_readfirstlane(t >> 6);
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int key0 = kbase + (ps * NW + w) * KPP;
            pg[ps] = key0 < ic.kv_end ? bt[key0 >> p.logP] : 0;
        }
    }
    // The same page ids through the vector memory path, for the direct-load pipeline of wide items: lane ps of a
    // wave fetches the id of the wave's pass ps with one load, and take_pages() moves the ids into scalar registers
    // once the load has landed.  Scalar loads share their counter with LDS reads and return out of order, so a wave
    // with page ids in flight has to drain that counter completely at its next fragment read; vector loads retire
    // in order behind the direct loads of the same step, and the wait that ends the step covers them.
    int pgv;
    __device__ __forceinline__ void fetch_pages_v(const AttnParams& p, const ItemCtx& ic, int kbase, int t) {
        const int key0 = kbase + (((t & 63) % NPASS) * NW + (t >> 6)) * KPP;
        pgv = key0 < ic.kv_end ? ic.bt_row[key0 >> p.logP] : 0;
    }
    __device__ __forceinline__ void take_pages() {
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) pg[ps] = __builtin_amdgcn_readlane(pgv, ps);
    }

    // The lane's first LDS slot inside its group, and which of the pass's groups that is.  Slot l = (quad, key, chunk in
    // quad); with two groups per pass a lane owns slots l and l + 1 (l even: neighbouring chunks of one key row).
    __device__ __forceinline__ static int lane_slot(int t) { return GPP == 1 ? (t & 63) : 2 * (t & 31); }
    __device__ __forceinline__ static int lane_group(int t) { return GPP == 1 ? 0 : (t & 63) >> 5; }
    __device__ __forceinline__ static int lane_key(int t) { return lane_group(t) * KPW + (lane_slot(t) >> 2) % KPW; }   // within the pass
    __device__ __forceinline__ static uint32_t lane_off(int t) {
        const int l = lane_slot(t);
        return (uint32_t)((lane_key(t) * D + ((l / (4 * KPW)) * 4 + (l & 3)) * 8) * ES);
    }

    struct Row {
        const char *kb, *vb;
        int key0, page;
    };
    __device__ __forceinline__ Row row_of(const AttnParams& p, const ItemCtx& ic, int kbase, int t, int ps) const {
        Row r;
        r.key0 = __builtin_amdgcn_readfirstlane(kbase + (ps * NW + (t >> 6)) * KPP);
        r.page = __builtin_amdgcn_readfirstlane(pg[ps]);
        const int64_t row = ((((int64_t)r.page * p.Hkv + ic.kvh) << p.logP) + (r.key0 & (p.P - 1))) * D * ES;
        r.kb = static_cast<const char*>(p.k_pool) + row;
        r.vb = static_cast<const char*>(p.v_pool) + row;
        return r;
    }
    // The same group when its keys are new tokens of this call: packed rows [token][Hkv][D] of k_new / v_new (bf16
    // cache only).  The base is the row of the group's first key (for a group that straddles C it lies before the
    // request's first row and is only ever used by lanes whose key is >= C); consecutive keys are Hkv rows apart.
    __device__ __forceinline__ Row new_row_of(const AttnParams& p, const ItemCtx& ic, const Row& r) const {
        Row n = r;
        const int64_t off = (((int64_t)ic.row_off + (r.key0 - ic.C)) * p.Hkv + ic.kvh) * (D * 2);
        n.kb = reinterpret_cast<const char*>(reinterpret_cast<intptr_t>(p.k_new) + off);
        n.vb = reinterpret_cast<const char*>(reinterpret_cast<intptr_t>(p.v_new) + off);
        return n;
    }
    __device__ __forceinline__ static uint32_t new_lane_off(const AttnParams& p, int t) {
        const int l = t & 63;
        return (uint32_t)(((l >> 2) % KPW) * p.Hkv * D * 2 + ((l / (4 * KPW)) * 4 + (l & 3)) * 16);
    }

    // ---- register-staged path
    // FULL: the whole tile lies inside the key range and in the pages
    template <bool FULL>
    __device__ __forceinline__ void fetch_kv_impl(const AttnParams& p, const ItemCtx& ic, int kbase, int t) {
        const uint32_t lo = lane_off(t);
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const Row r = row_of(p, ic, kbase, t, ps);
            // the scale slot this pass fills: its own, or (two scales) slot 0 from the first pass and slot 1 from the pass
            // of key 16, the first of the second page when pages hold 16 keys (with larger pages slot 1 is never read)
            const int sl = !TWO_SCALES ? ps : ps == 0 ? 0 : ps == 16 / KPP ? 1 : -1;
            if (sl >= 0) {
                ks[sl] = 1.0f;
                vs[sl] = 1.0f;
                if (KVT == KV_FP8 && (FULL || r.key0 < ic.kv_end)) {   // (a group past the key range has no page)
                    ks[sl] = p.k_scale[(int64_t)r.page * p.Hkv + ic.kvh];
                    vs[sl] = p.v_scale[(int64_t)r.page * p.Hkv + ic.kvh];
                }
            }
            const int key = r.key0 + lane_key(t);
            if (FULL || (key < ic.kv_end && key < ic.c_rows)) {
                k[ps].load(r.kb, lo);
                v[ps].load(r.vb, lo);
            } else if (KVT == KV_BF16 && key < ic.kv_end) {      // a new token of this call: read its packed row
                const Row n = new_row_of(p, ic, r);
                const uint32_t nlo = new_lane_off(p, t);
                k[ps].load(n.kb, nlo);
                v[ps].load(n.vb, nlo);
            } else {
                k[ps].zero();                                    // keys past the item's end: zeros, so
                v[ps].zero();                                    // that 0-weights never meet NaN garbage
            }
        }
    }
    __device__ __forceinline__ void fetch_kv(const AttnParams& p, const ItemCtx& ic, int kbase, int t) {
        if (kbase + NKEYS <= min(ic.kv_end, ic.c_rows))          // uniform: whole tile inside the key range, in pages
            fetch_kv_impl<true>(p, ic, kbase, t);
        else
            fetch_kv_impl<false>(p, ic, kbase, t);
    }
    // kl / vl: LDS byte addresses of this tile's K and V
    __device__ __forceinline__ void commit(const AttnParams& p, uint32_t kl, uint32_t vl, int t) const {
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const uint32_t o = ((ps * NW + (t >> 6)) * GPP + lane_group(t)) * G_::GS + lane_slot(t) * 16;
            if constexpr (KVT == KV_FP8) {
                *LDS_PTR(u32x4, kl + o) = k[ps].widen_first(k_scale_of(p, ps));
                *LDS_PTR(u32x4, kl + o + 16) = k[ps].widen_second(k_scale_of(p, ps));
                *LDS_PTR(u32x4, vl + o) = v[ps].widen_first(v_scale_of(p, ps));
                *LDS_PTR(u32x4, vl + o + 16) = v[ps].widen_second(v_scale_of(p, ps));
            } else {
                *LDS_PTR(u32x4, kl + o) = k[ps].widen(k_scale_of(p, ps));
                *LDS_PTR(u32x4, vl + o) = v[ps].widen(v_scale_of(p, ps));
            }
        }
    }

    // ---- direct path (bf16 only)
    template <bool FULL>
    __device__ __forceinline__ void dma_impl(const AttnParams& p, const ItemCtx& ic, int kbase, int t, uint32_t kl,
                                             uint32_t vl) const {
        const uint32_t lo = lane_off(t);
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const Row r = row_of(p, ic, kbase, t, ps);
            // wave-uniform LDS offset of the group
            const uint32_t go = __builtin_amdgcn_readfirstlane((ps * NW + (t >> 6)) * G_::GS);
            const int key = r.key0 + lane_key(t);
            if (FULL || (key < ic.kv_end && key < ic.c_rows)) {
                dma16(r.kb, lo, __builtin_amdgcn_readfirstlane(kl) + go);
                dma16(r.vb, lo, __builtin_amdgcn_readfirstlane(vl) + go);
            } else if (key < ic.kv_end) {                        // a new token of this call: its packed row
                const Row n = new_row_of(p, ic, r);
                const uint32_t nlo = new_lane_off(p, t);
                dma16(n.kb, nlo, __builtin_amdgcn_readfirstlane(kl) + go);
                dma16(n.vb, nlo, __builtin_amdgcn_readfirstlane(vl) + go);
            } else {
                *LDS_PTR(u32x4, kl + go + (t & 63) * 16) = u32x4{0, 0, 0, 0};
                *LDS_PTR(u32x4, vl + go + (t & 63) * 16) = u32x4{0, 0, 0, 0};
            }
        }
    }
    __device__ __forceinline__ void dma(const AttnParams& p, const ItemCtx& ic, int kbase, int t, uint32_t kl,
                                        uint32_t vl) const {
        if (kbase + NKEYS <= min(ic.kv_end, ic.c_rows))
            dma_impl<true>(p, ic, kbase, t, kl, vl);
        else
            dma_impl<false>(p, ic, kbase, t, kl, vl);
    }
};

// Final write of one wave's O^T: either bf16 output rows or fp32 partials.
//   row_in_item: this lane's row index inside the item (token_local * gn + head) or -1
template <int D>
__device__ __forceinline__ void store_result(const AttnParams& p, const ItemCtx& ic, WaveAcc<D>& st,
                                             int tok, int head_in_group, int row_in_item, int lane) {
    using G_ = Geo<D>;
    const int g = lane >> 5;
    const float ltot = sum_xor32(st.l);
    if (row_in_item < 0) return;
    if (ic.part_off < 0) {
        const float inv = 1.0f / ltot;
        const int hq = ic.kvh * (p.Hq / p.Hkv) + ic.g0 + head_in_group;
        char* dst = static_cast<char*>(p.out) + (((int64_t)(ic.row_off + tok) * p.Hq + hq) * D) * 2;
#pragma unroll
        for (int db = 0; db < G_::NDB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int d0 = db * 32 + i4 * 8 + g * 4;
                bf16x4 o = {(__bf16)(st.O[db][i4 * 4] * inv), (__bf16)(st.O[db][i4 * 4 + 1] * inv),
                            (__bf16)(st.O[db][i4 * 4 + 2] * inv), (__bf16)(st.O[db][i4 * 4 + 3] * inv)};
                *reinterpret_cast<u32x2*>(dst + d0 * 2) = __builtin_bit_cast(u32x2, o);
            }
    } else {
        const int rows = ic.nq * ic.gn;
        float* po = p.partial + ic.part_off + (int64_t)row_in_item * D;
#pragma unroll
        for (int db = 0; db < G_::NDB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int d0 = db * 32 + i4 * 8 + g * 4;
                f32x4 o = {st.O[db][i4 * 4], st.O[db][i4 * 4 + 1], st.O[db][i4 * 4 + 2], st.O[db][i4 * 4 + 3]};
                *reinterpret_cast<f32x4*>(po + d0) = o;
            }
        if (g == 0) {
            float* ml = p.partial + ic.part_off + (int64_t)rows * D + row_in_item * 2;
            ml[0] = st.m;
            ml[1] = ltot;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// wide body: 8 waves x 32 query rows share 128-key K/V stages (two in LDS: one consumed, one being filled).
// bf16 cache: stages travel global -> LDS directly, issued by one wave of every SIMD; one barrier per stage.
// 8-bit cache: register-staged and widened on the way into LDS, by all waves.

template <int D, int KVT>
__device__ __forceinline__ void wide_body(const AttnParams& p, const ItemCtx& ic, uint32_t smem, int tid) {
    using G_ = Geo<D>;
    constexpr bool DMA = KVT == KV_BF16;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tqw = 32 / ic.gn;                            // tokens per wave
    const int row = lane & 31;
    const int tl = row / ic.gn, hg = row - tl * ic.gn;
    const int tok_local = wave * tqw + tl;                 // token index inside the item
    const bool valid = tl < tqw && tok_local < ic.nq;
    const int tok = ic.q0 + tok_local;
    // wave-level causal bounds (last visible key = C + token)
    const int w_last = ic.C + ic.q0 + min(wave * tqw + tqw, ic.nq) - 1;
    const bool wave_active = wave * tqw < ic.nq;
    const int lim = valid ? ic.C + tok : 0x3fffffff;

    bf16x8 Q[G_::NKK];
    load_q<D>(p, ic, tok, hg, valid, lane, Q);
    WaveAcc<D> st;
#pragma unroll
    for (int db = 0; db < G_::NDB; ++db) st.O[db] = f32x16{0};
    st.m = NEG_INF;
    st.l = 0.0f;

    const int k_lo = ic.kv_begin;                          // multiple of 64
    const int ntiles = (ic.kv_end - k_lo + KT - 1) / KT;
    const int nfull = (ic.kv_end - k_lo) / KT;             // tiles 0..nfull-1 lie entirely inside the key range
    // Tiles whose last key is visible to every row of the workgroup need no causal select;
    // the remaining (at most a few) tiles around the diagonal take the masked variant.
    const int wg_first = ic.C + ic.q0;                     // smallest last-visible key in the workgroup
    const int t_diag = min(min(ntiles, nfull), max(0, (wg_first + 1 - k_lo) / KT));   // (a ragged last stage is masked too)
    Loader<D, KVT, AWG, KT> ld;
    PipeState<D> ps;
    // keys from kv_end on (the ragged tail of the last stage) count as masked
    const int lim_eff = min(lim, ic.kv_end - 1);
    // a wave without rows, or one whose rows all end before this stage, skips it
    auto computes = [&](int t) { return wave_active && k_lo + t * KT <= w_last; };
    auto compute = [&](int t, uint32_t stage, auto masked) {
        const int kbase = k_lo + t * KT;
        if (computes(t))
            stage_pipelined<D, decltype(masked)::value>(stage, stage + G_::KTILE, Q, st, ps, p.c_log2,
                                                        lim_eff - kbase - 4 * (lane >> 5), lane);
    };
    if (DMA) {
        // Who issues the direct loads.  The CU's memory pipeline takes one 1 KB direct load every ~23 cycles, and a
        // wave whose load finds the queue full is blocked (instructions issue in order) and computes nothing: when all
        // eight waves issued their share at the start of a stage, the matrix pipes of all four SIMDs stood still for
        // the ~1 500 cycles the 64 loads of a stage need, in every stage.  So only one wave of every SIMD loads (waves
        // w and w + 4 share a SIMD): the four loading waves issue the whole next stage at the start of a stage while
        // their SIMD partners already compute, and catch up afterwards.  A tile with rows for at most four waves lets
        // its idle half do the loading.
        static_assert(NSTAGE == 2, "tile t + 1 is loaded during stage t; the page ids of tile t + 2 travel behind it");
        constexpr int LW = ATTN_WAVES / 2;
        using LD = Loader<D, KVT, 64 * LW, KT>;
        LD ldh;
        const int n_active = (ic.nq + tqw - 1) / tqw;      // waves that have rows
        const int lbase = n_active <= LW ? LW : 0;
        const bool loader = wave >= lbase && wave < lbase + LW;
        const int lt = tid - lbase * 64;                   // thread index among the loading waves
        if (loader) {
            ldh.fetch_pages(p, ic, k_lo, lt);
            ldh.dma(p, ic, k_lo, lt, smem, smem + G_::KTILE);
            if (ntiles > 1) ldh.fetch_pages_v(p, ic, k_lo + KT, lt);
        }
        dma_wait();
        __syncthreads();
        auto step = [&](int t, auto masked) {
            if (loader && t + 1 < ntiles) {
                const uint32_t sg = smem + ((t + 1) % NSTAGE) * G_::WIDE_STAGE;
                ldh.take_pages();                          // (their load was waited for at the end of the previous step)
                ldh.dma(p, ic, k_lo + (t + 1) * KT, lt, sg, sg + G_::KTILE);
                if (t + 2 < ntiles) ldh.fetch_pages_v(p, ic, k_lo + (t + 2) * KT, lt);
            }
            compute(t, smem + (t % NSTAGE) * G_::WIDE_STAGE, masked);
            dma_wait();                                    // tile t+1 and the page ids of tile t+2 have landed
            __syncthreads();
        };
        for (int t = 0; t < t_diag; ++t) step(t, std::false_type{});
        for (int t = t_diag; t < ntiles; ++t) step(t, std::true_type{});
    } else {
        static_assert(NSTAGE >= 2, "two stages for the register-staged path");
        ld.fetch_pages(p, ic, k_lo, tid);
        ld.fetch_kv(p, ic, k_lo, tid);
        if (ntiles > 1) ld.fetch_pages(p, ic, k_lo + KT, tid);
        ld.commit(p, smem, smem + G_::KTILE, tid);
        __syncthreads();
        auto step = [&](int t, auto masked) {
            const uint32_t cur = smem + (t & 1) * G_::WIDE_STAGE;
            const uint32_t nxt = smem + ((t + 1) & 1) * G_::WIDE_STAGE;
            const bool more = t + 1 < ntiles;
            if (more) {
                ld.fetch_kv(p, ic, k_lo + (t + 1) * KT, tid);
                if (t + 2 < ntiles) ld.fetch_pages(p, ic, k_lo + (t + 2) * KT, tid);
            }
            compute(t, cur, masked);
            if (more) ld.commit(p, nxt, nxt + G_::KTILE, tid);
            __syncthreads();
        };
        for (int t = 0; t < t_diag; ++t) step(t, std::false_type{});
        for (int t = t_diag; t < ntiles; ++t) step(t, std::true_type{});
    }
    store_result<D>(p, ic, st, tok, hg, valid ? tok_local * ic.gn + hg : -1, lane);
}

// ---------------------------------------------------------------------------------------------
// narrow body: <= 32 query rows; the 8 waves take 32-key blocks round-robin, each through its
// own LDS region, and merge their (m, l, O) through LDS at the end

// ROWS: query rows a wave carries (32, or 16 for items of at most 16 rows: half the matrix and softmax work per key)
template <int D, int KVT, int ROWS>
__device__ __forceinline__ void narrow_body(const AttnParams& p, const ItemCtx& ic, uint32_t smem, int tid) {
    using G_ = Geo<D>;
    constexpr bool R16 = ROWS == 16;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row = lane & (ROWS - 1);
    const int tl = row / ic.gn, hg = row - tl * ic.gn;
    const bool valid = tl < ic.nq;
    const int tok = ic.q0 + tl;
    const int lim = valid ? ic.C + tok : 0x3fffffff;
    const int first_lim = ic.C + ic.q0;                  // smallest last-visible key among the rows

    bf16x8 Q[R16 ? D / 32 : G_::NKK];
    std::conditional_t<R16, WaveAcc16<D>, WaveAcc<D>> st;
    if constexpr (R16) {
        load_q16<D>(p, ic, tok, hg, valid, lane, Q);
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) st.O[dt] = f32x4{0, 0, 0, 0};
    } else {
        load_q<D>(p, ic, tok, hg, valid, lane, Q);
#pragma unroll
        for (int db = 0; db < G_::NDB; ++db) st.O[db] = f32x16{0};
    }
    st.m = NEG_INF;
    st.l = 0.0f;

    const uint32_t kl = smem + wave * (2 * G_::B32);
    const uint32_t vl = kl + G_::B32;
    const int nblocks = (ic.kv_end - ic.kv_begin + 31) >> 5;
    Loader<D, KVT, 64, 32> ld;
    if (wave < nblocks) {
        ld.fetch_pages(p, ic, ic.kv_begin + wave * 32, lane);
        ld.fetch_kv(p, ic, ic.kv_begin + wave * 32, lane);
        if (wave + ATTN_WAVES < nblocks) ld.fetch_pages(p, ic, ic.kv_begin + (wave + ATTN_WAVES) * 32, lane);
    }
    for (int b = wave; b < nblocks; b += ATTN_WAVES) {
        const int kbase = ic.kv_begin + b * 32;
        ld.commit(p, kl, vl, lane);
        if (b + ATTN_WAVES < nblocks) {
            ld.fetch_kv(p, ic, kbase + 32 * ATTN_WAVES, lane);
            if (b + 2 * ATTN_WAVES < nblocks) ld.fetch_pages(p, ic, kbase + 64 * ATTN_WAVES, lane);
        }
        if constexpr (R16)
            block16<D>(kl, vl, Q, st, p.c_log2, lim - kbase - 4 * key_group16(lane >> 4), kbase + 31 > first_lim, lane);
        else
            block32<D>(kl, vl, Q, st, p.c_log2, lim - kbase - 4 * (lane >> 5), kbase + 31 > first_lim, lane);
    }
    // merge the waves: LDS holds O as [wave][row 0..31][D + 4] fp32 and (m, l) as [wave][32][2]
    const float ltot = R16 ? sum_xor32(sum_xor16(st.l)) : sum_xor32(st.l);
    __syncthreads();                                      // every wave is done with its K/V region
    constexpr int NW = ATTN_WAVES;
    constexpr int OSTR = D + 4;
    const uint32_t obase = smem;
    const uint32_t mlbase = smem + NW * 32 * OSTR * 4;
    {
        const int g = lane / ROWS;
        const uint32_t orow = obase + ((wave * 32 + row) * OSTR) * 4;
        if constexpr (R16) {
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt) *LDS_PTR(f32x4, orow + (dt * 16 + g * 4) * 4) = st.O[dt];
        } else {
#pragma unroll
            for (int db = 0; db < G_::NDB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const int d0 = db * 32 + i4 * 8 + g * 4;
                    f32x4 o = {st.O[db][i4 * 4], st.O[db][i4 * 4 + 1], st.O[db][i4 * 4 + 2], st.O[db][i4 * 4 + 3]};
                    *LDS_PTR(f32x4, orow + d0 * 4) = o;
                }
        }
        if (g == 0) {
            *LDS_PTR(float, mlbase + ((wave * 32 + row) * 2) * 4) = st.m;
            *LDS_PTR(float, mlbase + ((wave * 32 + row) * 2 + 1) * 4) = ltot;
        }
    }
    __syncthreads();
    // thread -> (row r, DPT consecutive d): 16 threads per row
    constexpr int DPT = D / 16;
    const int r = tid >> 4, dc = (tid & 15) * DPT;
    const int rows = ic.nq * ic.gn;
    if (r < rows) {
        float mw[NW], lw[NW];
        float mall = NEG_INF;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            mw[w] = *LDS_PTR(float, mlbase + ((w * 32 + r) * 2) * 4);
            lw[w] = *LDS_PTR(float, mlbase + ((w * 32 + r) * 2 + 1) * 4);
            mall = fmaxf(mall, mw[w]);
        }
        const float muse = mall == NEG_INF ? 0.0f : mall;
        float lsum = 0.0f, wgt[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            wgt[w] = fast_exp2(mw[w] - muse);
            lsum += lw[w] * wgt[w];
        }
        float acc[DPT];
#pragma unroll
        for (int x = 0; x < DPT; ++x) acc[x] = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const uint32_t src = obase + ((w * 32 + r) * OSTR + dc) * 4;
#pragma unroll
            for (int x = 0; x < DPT; x += 4) {
                const f32x4 o = *LDS_PTR(f32x4, src + x * 4);
                acc[x] += o[0] * wgt[w];
                acc[x + 1] += o[1] * wgt[w];
                acc[x + 2] += o[2] * wgt[w];
                acc[x + 3] += o[3] * wgt[w];
            }
        }
        const int rtl = r / ic.gn, rhg = r - rtl * ic.gn;
        if (ic.part_off < 0) {
            const float inv = 1.0f / lsum;
            const int hq = ic.kvh * (p.Hq / p.Hkv) + ic.g0 + rhg;
            char* dst = static_cast<char*>(p.out) + (((int64_t)(ic.row_off + ic.q0 + rtl) * p.Hq + hq) * D + dc) * 2;
#pragma unroll
            for (int x = 0; x < DPT; x += 4) {
                bf16x4 o = {(__bf16)(acc[x] * inv), (__bf16)(acc[x + 1] * inv), (__bf16)(acc[x + 2] * inv),
                            (__bf16)(acc[x + 3] * inv)};
                *reinterpret_cast<u32x2*>(dst + x * 2) = __builtin_bit_cast(u32x2, o);
            }
        } else {
            float* po = p.partial + ic.part_off + (int64_t)r * D + dc;
#pragma unroll
            for (int x = 0; x < DPT; x += 4) {
                f32x4 o = {acc[x], acc[x + 1], acc[x + 2], acc[x + 3]};
                *reinterpret_cast<f32x4*>(po + x) = o;
            }
            if ((tid & 15) == 0) {
                float* ml = p.partial + ic.part_off + (int64_t)rows * D + r * 2;
                ml[0] = mall;
                ml[1] = lsum;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// append item (bf16 cache): the page writes of the call, riding in the attention launch.  One item moves nq
// consecutive packed rows of k_new / v_new, starting with new token q0 of request req and running on into the
// following requests, to their pages: a bit-exact copy, 16 bytes per thread and step.  The attention items of
// the same launch never read these page slots (they take new tokens from the packed rows), so the two kinds
// need no order among themselves.

__device__ __forceinline__ void append_body(const AttnParams& p, const ItemCtx& ic, int D, int tid) {
    const int cpt = p.Hkv * D / 8;                           // 16-byte chunks per packed row (one of K or V)
    const int cph = D / 8;
    const int first_row = ic.row_off + ic.q0;                // packed row of the item's first token
    const int total = ic.nq * cpt;
    int r = ic.req;                                          // request of the row this thread is at: rows only move forward
    ReqInfo ri = p.reqs[r];
    for (int u = tid; u < total; u += AWG) {
        const int row = first_row + u / cpt, rem = u % cpt;
        while (row >= ri.row_off + ri.L) ri = p.reqs[++r];   // (requests with L = 0 are stepped over)
        const int h = rem / cph, ch = rem % cph;
        const int t = ri.C + (row - ri.row_off);
        const int page = p.block_table[(int64_t)r * p.max_pages + (t >> p.logP)];
        const int64_t src = ((int64_t)row * p.Hkv + h) * D + ch * 8;
        const int64_t dst = ((((int64_t)page * p.Hkv + h) << p.logP) + (t & (p.P - 1))) * D + ch * 8;
        const u32x4 kx = *reinterpret_cast<const u32x4*>(static_cast<const char*>(p.k_new) + src * 2);
        const u32x4 vx = *reinterpret_cast<const u32x4*>(static_cast<const char*>(p.v_new) + src * 2);
        *reinterpret_cast<u32x4*>(static_cast<char*>(const_cast<void*>(p.k_pool)) + dst * 2) = kx;
        *reinterpret_cast<u32x4*>(static_cast<char*>(const_cast<void*>(p.v_pool)) + dst * 2) = vx;
    }
}

// ---------------------------------------------------------------------------------------------
// the fused attention launch: one workgroup per work item, wide and narrow items in one grid

// Next item of die queue q (items q, q + NUM_QUEUES, ...), or -1 when the queue is used up.
__device__ __forceinline__ int take_item(const AttnParams& p, int q) {
    const int pos = __hip_atomic_fetch_add(p.queue_heads + q, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int idx = q + NUM_QUEUES * pos;
    return idx < p.nitems ? idx : -1;
}
// An item of the queue with the most items left, or -1 when every queue is used up.  Called by the whole first wave: lanes
// 0 .. NUM_QUEUES - 1 read one queue head each (one round trip for the scan), lane 0 takes the item.  Bounded: an attempt
// fails only when another workgroup took the last item of the chosen queue in between, and that workgroup runs it.
__device__ __forceinline__ int steal_item(const AttnParams& p, int lane) {
    for (int attempt = 0; attempt < 4 * NUM_QUEUES; ++attempt) {
        int left = 0;
        if (lane < NUM_QUEUES) {
            const int pos = __hip_atomic_load(p.queue_heads + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            left = (p.nitems - lane + NUM_QUEUES - 1) / NUM_QUEUES - pos;
        }
        int best = -1, best_left = 0;
#pragma unroll
        for (int q = 0; q < NUM_QUEUES; ++q) {
            const int l = __builtin_amdgcn_readlane(left, q);
            if (l > best_left) {
                best_left = l;
                best = q;
            }
        }
        if (best < 0) return -1;
        int idx = -1;
        if (lane == 0) idx = take_item(p, best);
        idx = __builtin_amdgcn_readfirstlane(idx);
        if (idx >= 0) return idx;
    }
    return -1;
}

template <int D, int KVT>
__device__ __forceinline__ void run_item(const AttnParams& p, int idx, uint32_t smem, int tid) {
    const int kind = (p.items[idx].heads >> 24) & 0xff;
    if (kind == KIND_NULL) return;                         // a filler that keeps the following items on their XCD
    const ItemCtx ic = load_item(p, idx);
    if (kind == KIND_WIDE)
        wide_body<D, KVT>(p, ic, smem, tid);
    else if (kind == KIND_NARROW) {
        if (ic.nq * ic.gn <= 16)
            narrow_body<D, KVT, 16>(p, ic, smem, tid);
        else
            narrow_body<D, KVT, 32>(p, ic, smem, tid);
    }
    else if (KVT == KV_BF16)
        append_body(p, ic, D, tid);
}

// One workgroup per work item when the items fit one round on the CUs (gridDim.x = number of items).  Otherwise
// gridDim.x persistent workgroups: workgroup i runs item i, then items of the queue of its die (workgroup i of a launch
// is dispatched to die i % NUM_QUEUES, and so were the items of queue i % NUM_QUEUES meant to be: their K/V streams share
// that die's L2), and when that queue is used up it helps out on the queue with the most items left, so that the dies
// finish together.
// No workgroup ever waits for another: every loop ends when the queues are used up.
template <int D, int KVT>
__global__ __launch_bounds__(AWG, 1) void attn_kernel(const AttnParams p) {
    __shared__ __attribute__((aligned(16))) char smem_raw[Geo<D>::SMEM];
    __shared__ int s_next;
    const uint32_t smem = (uint32_t)(uintptr_t)LDS_PTR(char, smem_raw);
    if (blockIdx.x == 0 && threadIdx.x == 0 && p.slot_flag)   // releases the host's staging slot (see AttnParams)
        __hip_atomic_store(p.slot_flag, p.slot_seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    const bool persistent = p.nitems > (int)gridDim.x;
    const int home = blockIdx.x % NUM_QUEUES;
    int idx = blockIdx.x;
    for (;;) {
        // The thread index is made opaque in every iteration: otherwise everything the three kinds of item derive from it
        // is hoisted out of the loop and live at once, which does not fit the register file (spills to scratch memory).
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        run_item<D, KVT>(p, idx, smem, tid);
        if (!persistent) return;
        __syncthreads();                                   // every wave is done with this item's LDS
        if (tid < 64) {
            // The next item is taken when this one is done, not before (measured: a reservation at the start of the item
            // +5 % on long tiles, one during its last stage +1 %): the queues are ordered longest first, and an item
            // reserved early goes to a workgroup by its position in the launch instead of to the one that is free first.
            int next = -1;
            if (tid == 0) next = take_item(p, home);
            next = __builtin_amdgcn_readfirstlane(next);
            if (next < 0) next = steal_item(p, tid);
            if (tid == 0) s_next = next;
        }
        __syncthreads();
        idx = __builtin_amdgcn_readfirstlane(s_next);      // uniform: the item is then read through the scalar unit
        __syncthreads();                                   // (s_next is written again at the end of the next item)
        if (idx < 0) return;
    }
}

// ---------------------------------------------------------------------------------------------
// combine: merge the split-KV partials of one query tile
//   m = max_s m_s;  l = sum_s l_s 2^(m_s - m);  O = sum_s O_s 2^(m_s - m) / l

constexpr int COMB_ROWS = 16;          // query rows per combine workgroup when a tile has few splits
constexpr int COMB_ROWS_SLICED = 2;    // ... and when it has many: the workgroup's threads then share the splits

// One output quad (4 consecutive d of one row) merged over the splits s_begin, s_begin + s_step, ... < nsplit, UN splits
// at a time: all loads of a group are issued before any is used, so a thread pays one memory latency per UN splits,
// and the maximum is carried along (acc and l are rescaled when a group raises it) instead of being taken in a pass
// of its own.  Returns the running maximum (-inf when the thread had no split).
template <int D, int UN>
__device__ __forceinline__ float combine_quad(const float* part0, int nsplit, int s_begin, int s_step, int64_t stride,
                                              int64_t ml_off, int64_t o_off, f32x4& acc, float& lsum) {
    float m_run = NEG_INF;
    lsum = 0.0f;
    acc = f32x4{0, 0, 0, 0};
    for (int s0 = s_begin; s0 < nsplit; s0 += UN * s_step) {
        float mv[UN], lv[UN];
        f32x4 ov[UN];
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const int sp = min(s0 + j * s_step, nsplit - 1);         // the tail re-reads the last split and drops it below
            const float* base = part0 + (int64_t)sp * stride;
            mv[j] = base[ml_off];
            lv[j] = base[ml_off + 1];
            ov[j] = *reinterpret_cast<const f32x4*>(base + o_off);
        }
        float mg = m_run;
#pragma unroll
        for (int j = 0; j < UN; ++j) mg = fmaxf(mg, mv[j]);          // (a duplicate of the last split changes nothing)
        const float muse = mg == NEG_INF ? 0.0f : mg;
        const float back = fast_exp2(m_run - muse);                  // 0 on the first group
        lsum *= back;
        acc *= back;
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            if (s0 + j * s_step < nsplit) {
                const float w = fast_exp2(mv[j] - muse);
                lsum += lv[j] * w;
                acc += ov[j] * w;
            }
        }
        m_run = mg;
    }
    return m_run;
}

// CR query rows per workgroup.  CR * D / 4 output quads; when that is less than the workgroup, its WG / (CR * D / 4)
// thread slices each take every NSL-th split of a quad and slice 0 merges their results through LDS: a tile with a
// hundred splits and few rows (a decode row over a long context) is then a chain of one or two memory latencies per
// thread instead of eight, on NSL times as many workgroups.
template <int D, int CR>
__global__ __launch_bounds__(WG) void combine_kernel(const AttnParams p) {
    constexpr int QPR = D / 4;                         // float4 groups per row
    constexpr int NSL = CR * QPR >= WG ? 1 : WG / (CR * QPR);
    constexpr int PER = CR * QPR < WG ? CR * QPR : WG; // (row, quad) pairs in flight per pass
    __shared__ float red[NSL > 1 ? (NSL - 1) * PER * 6 : 1];
    const CombItem ci = p.combs[blockIdx.x];
    const int kvh = ci.heads & 0xff, g0 = (ci.heads >> 8) & 0xff, gn = (ci.heads >> 16) & 0xff;
    const int rows = ci.nq * gn;
    const int r0 = blockIdx.y * CR;                    // grid.y covers the tallest tile
    if (r0 >= rows) return;
    const ReqInfo ri = p.reqs[ci.req];
    const int nr = min(CR, rows - r0);
    const int slice = threadIdx.x / PER, u0 = threadIdx.x % PER;
    const float* part0 = p.partial + ci.part_off;
    auto finish = [&](int r, int dq, const f32x4& acc, float lsum) {
        const float inv = 1.0f / lsum;
        const int tl = r / gn, hg = r - tl * gn;
        const int hq = kvh * (p.Hq / p.Hkv) + g0 + hg;
        char* dst = static_cast<char*>(p.out) + (((int64_t)(ri.row_off + ci.q0 + tl) * p.Hq + hq) * D + dq) * 2;
        bf16x4 o = {(__bf16)(acc[0] * inv), (__bf16)(acc[1] * inv), (__bf16)(acc[2] * inv), (__bf16)(acc[3] * inv)};
        *reinterpret_cast<u32x2*>(dst) = __builtin_bit_cast(u32x2, o);
    };
    if constexpr (NSL == 1) {
        for (int u = u0; u < nr * QPR; u += PER) {
            const int r = r0 + u / QPR, dq = (u % QPR) * 4;
            const int64_t ml_off = (int64_t)rows * D + r * 2;
            float lsum;
            f32x4 acc;
            if (ci.nsplit > 8)
                combine_quad<D, 16>(part0, ci.nsplit, 0, 1, ci.part_stride, ml_off, (int64_t)r * D + dq, acc, lsum);
            else
                combine_quad<D, 4>(part0, ci.nsplit, 0, 1, ci.part_stride, ml_off, (int64_t)r * D + dq, acc, lsum);
            finish(r, dq, acc, lsum);
        }
    } else {
        const bool active = u0 < nr * QPR;             // one pass: nr * QPR <= PER
        const int r = r0 + u0 / QPR, dq = (u0 % QPR) * 4;
        float lsum = 0.0f, m = NEG_INF;
        f32x4 acc = {0, 0, 0, 0};
        if (active)
            m = combine_quad<D, 16>(part0, ci.nsplit, slice, NSL, ci.part_stride, (int64_t)rows * D + r * 2,
                                    (int64_t)r * D + dq, acc, lsum);
        if (active && slice > 0) {
            float* w = red + ((slice - 1) * PER + u0) * 6;
            w[0] = m; w[1] = lsum; w[2] = acc[0]; w[3] = acc[1]; w[4] = acc[2]; w[5] = acc[3];
        }
        __syncthreads();
        if (!active || slice > 0) return;
        float mall = m;
#pragma unroll
        for (int s = 1; s < NSL; ++s) mall = fmaxf(mall, red[((s - 1) * PER + u0) * 6]);
        const float muse = mall == NEG_INF ? 0.0f : mall;
        const float w0 = fast_exp2(m - muse);
        lsum *= w0;
        acc *= w0;
#pragma unroll
        for (int s = 1; s < NSL; ++s) {
            const float* rd = red + ((s - 1) * PER + u0) * 6;
            const float w = fast_exp2(rd[0] - muse);
            lsum += rd[1] * w;
            acc += f32x4{rd[2], rd[3], rd[4], rd[5]} * w;
        }
        finish(r, dq, acc, lsum);
    }
}

// ---------------------------------------------------------------------------------------------
// KV append / pack / unpack, bf16 cache: bit-exact copies.  grid = (pages touched, requests, 2 {K,V})

// The z-slice past the K / V slices of an append launch carries the work list of the attention launch
// that follows from pinned host memory into the workspace (saves a launch per call).
__device__ __forceinline__ void upload_rider(const AppendParams& p) {
    const u32x4* src = static_cast<const u32x4*>(p.up_src);
    u32x4* dst = static_cast<u32x4*>(p.up_dst);
    const int nthreads = gridDim.x * gridDim.y * WG;
    for (int i = (blockIdx.y * gridDim.x + blockIdx.x) * WG + threadIdx.x; i < p.up_n16; i += nthreads) dst[i] = src[i];
}

// PACK = false: packed rows [tokens][hn][D] -> pages (append, or unpack of a received head share);
// PACK = true:  pages -> packed rows (the send buffer of a KV transfer).
template <bool PACK>
__global__ __launch_bounds__(WG) void kv_move_bf16_kernel(const AppendParams p) {
    if (blockIdx.z == 2) {
        upload_rider(p);
        return;
    }
    const int r = blockIdx.y;
    const int C = p.C[r], L = p.L[r];
    const int lp = (C >> p.logP) + blockIdx.x;               // logical page
    const int t0 = max(C, lp << p.logP), t1 = min(C + L, (lp + 1) << p.logP);
    if (t0 >= t1) return;
    const int page = p.block_table[(int64_t)(p.req0 + r) * p.max_pages + lp];
    const int cpt = p.hn * p.D / 8;                          // 16-byte chunks per packed token row
    const int cph = p.D / 8;
    char* rows = static_cast<char*>(const_cast<void*>(blockIdx.z ? p.v_new : p.k_new));
    char* pool = static_cast<char*>(blockIdx.z ? p.v_pool : p.k_pool);
    const int total = (t1 - t0) * cpt;
    for (int u = threadIdx.x; u < total; u += WG) {
        const int t = t0 + u / cpt, rem = u % cpt;
        const int h = rem / cph, ch = rem % cph;
        char* rp = rows + (((int64_t)(p.row_off[r] + t - C) * p.hn + h) * p.D + ch * 8) * 2;
        char* pp = pool + (((((int64_t)page * p.Hkv + p.h0 + h) << p.logP) + (t & (p.P - 1))) * p.D + ch * 8) * 2;
        if (PACK)
            *reinterpret_cast<u32x4*>(rp) = *reinterpret_cast<const u32x4*>(pp);
        else
            *reinterpret_cast<u32x4*>(pp) = *reinterpret_cast<const u32x4*>(rp);
    }
}

// KV append, 8-bit cache.  grid = (pages touched, requests, 2 {K,V} x KV heads): one block per
// (page, head), so that the chain amax of the new tokens -> exponent -> (re-encode old slots) -> encode,
// which is a few dependent memory round trips, runs for all heads at once.
__device__ __forceinline__ int exponent_for(float amax) {
    // smallest e with amax <= 448 * 2^e  (448 = 1.75 * 2^8), clamped to [-40, 119]
    const uint32_t u = __float_as_uint(amax);
    const int ex = (int)(u >> 23) - 127;
    const uint32_t man = u & 0x7fffffu;
    int e = (man <= 0x600000u) ? ex - 8 : ex - 7;
    if ((u >> 23) == 0) e = -40;                              // zero / subnormal
    return min(119, max(-40, e));
}

__device__ __forceinline__ uint32_t encode4(float a, float b, float c, float d) {
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
    return (uint32_t)w;
}

__global__ __launch_bounds__(WG) void append_fp8_kernel(const AppendParams p) {
    __shared__ float red[WG / 64];
    __shared__ int e_sh[2];
    if ((int)blockIdx.z == 2 * p.Hkv) {
        upload_rider(p);
        return;
    }
    const int r = blockIdx.y;
    const int C = p.C[r], L = p.L[r];
    const int lp = (C >> p.logP) + blockIdx.x;
    const int t0 = max(C, lp << p.logP), t1 = min(C + L, (lp + 1) << p.logP);
    if (t0 >= t1) return;
    const int page = p.block_table[(int64_t)(p.req0 + r) * p.max_pages + lp];
    const int n_old = max(0, C - (lp << p.logP));
    const int is_v = blockIdx.z & 1, h = blockIdx.z >> 1;
    const char* src = static_cast<const char*>(is_v ? p.v_new : p.k_new);
    uint8_t* dst = static_cast<uint8_t*>(is_v ? p.v_pool : p.k_pool);
    float* scl = is_v ? p.v_scale : p.k_scale;
    const int cph = p.D / 8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    {
        // 1. amax over the new tokens of this (page, head)
        float amax = 0.0f;
        const int total = (t1 - t0) * cph;
        for (int u = threadIdx.x; u < total; u += WG) {
            const int t = t0 + u / cph, ch = u % cph;
            const u32x4 v = *reinterpret_cast<const u32x4*>(src + (((int64_t)(p.row_off[r] + t - C) * p.Hkv + h) * p.D + ch * 8) * 2);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                amax = fmaxf(amax, fabsf(__uint_as_float(w[x] << 16)));
                amax = fmaxf(amax, fabsf(__uint_as_float(w[x] & 0xffff0000u)));
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
        if (lane == 0) red[wave] = amax;
        __syncthreads();
        if (threadIdx.x == 0) {
            float a = red[0];
            for (int w = 1; w < WG / 64; ++w) a = fmaxf(a, red[w]);
            int e = exponent_for(a);
            int e_old = e;
            if (n_old > 0) {
                const float s_old = scl[(int64_t)page * p.Hkv + h];
                e_old = (int)(__float_as_uint(s_old) >> 23) - 127;
                if (e < e_old) e = e_old;
            }
            e_sh[0] = e;
            e_sh[1] = e_old;
            scl[(int64_t)page * p.Hkv + h] = __uint_as_float((uint32_t)(e + 127) << 23);
        }
        __syncthreads();
        const int e = e_sh[0], e_old = e_sh[1];
        uint8_t* pg = dst + ((((int64_t)page * p.Hkv + h) << p.logP)) * p.D;
        // 2. re-encode the slots that were already valid when the exponent rises
        if (n_old > 0 && e > e_old) {
            const float f = __uint_as_float((uint32_t)(e_old - e + 127) << 23);     // 2^(e_old - e)
            const int tot_old = n_old * (p.D / 4);
            for (int u = threadIdx.x; u < tot_old; u += WG) {
                uint32_t* q4 = reinterpret_cast<uint32_t*>(pg) + u;
                const uint32_t w = *q4;
                const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(w, false);
                const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(w, true);
                *q4 = encode4(lo.x * f, lo.y * f, hi.x * f, hi.y * f);
            }
        }
        // 3. encode the new tokens: x * 2^-e, |.| <= 448 by construction
        const float inv = __uint_as_float((uint32_t)(127 - e) << 23);
        for (int u = threadIdx.x; u < total; u += WG) {
            const int t = t0 + u / cph, ch = u % cph;
            const u32x4 v = *reinterpret_cast<const u32x4*>(src + (((int64_t)(p.row_off[r] + t - C) * p.Hkv + h) * p.D + ch * 8) * 2);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            float f[8];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                f[2 * x] = __uint_as_float(w[x] << 16) * inv;
                f[2 * x + 1] = __uint_as_float(w[x] & 0xffff0000u) * inv;
            }
            u32x2 o;
            o.x = encode4(f[0], f[1], f[2], f[3]);
            o.y = encode4(f[4], f[5], f[6], f[7]);
            *reinterpret_cast<u32x2*>(pg + (int64_t)(t & (p.P - 1)) * p.D + ch * 8) = o;
        }
    }
}

// Work-list upload: the workgroups read the host-built plan straight out of pinned host memory
// and write it to the workspace (cheaper than a runtime copy command for ~100 KB).
__global__ __launch_bounds__(WG) void upload_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int n16) {
    const int i = blockIdx.x * WG + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

// ---------------------------------------------------------------------------------------------
// launchers

hipError_t launch_upload(const void* h_src, void* d_dst, size_t bytes, hipStream_t st) {
    const int n16 = (int)((bytes + 15) / 16);
    if (n16 <= 0) return hipSuccess;
    hipLaunchKernelGGL(upload_kernel, dim3((n16 + WG - 1) / WG), dim3(WG), 0, st,
                       static_cast<const u32x4*>(h_src), static_cast<u32x4*>(d_dst), n16);
    return hipGetLastError();
}

template <int D, int KVT>
static hipError_t launch_attn_t(const AttnParams& p, int grid, hipStream_t st) {
    hipLaunchKernelGGL((attn_kernel<D, KVT>), dim3(grid), dim3(AWG), 0, st, p);
    return hipGetLastError();
}

hipError_t launch_attn(const AttnParams& p, int D, int kvt, int grid, hipStream_t st) {
    if (grid <= 0) return hipSuccess;
    if (D == 128 && kvt == KV_BF16) return launch_attn_t<128, KV_BF16>(p, grid, st);
    if (D == 64 && kvt == KV_BF16) return launch_attn_t<64, KV_BF16>(p, grid, st);
    if (D == 128 && kvt == KV_FP8) return launch_attn_t<128, KV_FP8>(p, grid, st);
    if (D == 64 && kvt == KV_FP8) return launch_attn_t<64, KV_FP8>(p, grid, st);
    return hipErrorInvalidValue;
}

// max_rows: rows of the tallest tile; max_splits: splits of the most finely split one
hipError_t launch_combine(const AttnParams& p, int D, int ncombs, int max_rows, int max_splits, hipStream_t st) {
    if (ncombs <= 0) return hipSuccess;
    // many splits and a launch that would otherwise leave most of the chip idle: let thread slices share the splits
    const bool sliced = max_splits > 16 && (int64_t)ncombs * ((max_rows + COMB_ROWS - 1) / COMB_ROWS) < 512;
    const int cr = sliced ? COMB_ROWS_SLICED : COMB_ROWS;
    const dim3 grid(ncombs, (max_rows + cr - 1) / cr);
    if (D == 128) {
        if (sliced)
            hipLaunchKernelGGL((combine_kernel<128, COMB_ROWS_SLICED>), grid, dim3(WG), 0, st, p);
        else
            hipLaunchKernelGGL((combine_kernel<128, COMB_ROWS>), grid, dim3(WG), 0, st, p);
    } else {
        if (sliced)
            hipLaunchKernelGGL((combine_kernel<64, COMB_ROWS_SLICED>), grid, dim3(WG), 0, st, p);
        else
            hipLaunchKernelGGL((combine_kernel<64, COMB_ROWS>), grid, dim3(WG), 0, st, p);
    }
    return hipGetLastError();
}

hipError_t launch_append(const AppendParams& p, int kvt, int max_pages_touched, int nreq, hipStream_t st) {
    if (nreq <= 0 || max_pages_touched <= 0) return hipSuccess;               // (the caller keeps a rider for later)
    const int rider = p.up_n16 > 0 ? 1 : 0;
    if (kvt == KV_BF16)
        hipLaunchKernelGGL(kv_move_bf16_kernel<false>, dim3(max_pages_touched, nreq, 2 + rider), dim3(WG), 0, st, p);
    else
        hipLaunchKernelGGL(append_fp8_kernel, dim3(max_pages_touched, nreq, 2 * p.Hkv + rider), dim3(WG), 0, st, p);
    return hipGetLastError();
}

hipError_t launch_kv_move(const AppendParams& p, bool pack, int max_pages_touched, int nreq, hipStream_t st) {
    if (nreq <= 0 || max_pages_touched <= 0) return hipSuccess;
    if (pack)
        hipLaunchKernelGGL(kv_move_bf16_kernel<true>, dim3(max_pages_touched, nreq, 2), dim3(WG), 0, st, p);
    else
        hipLaunchKernelGGL(kv_move_bf16_kernel<false>, dim3(max_pages_touched, nreq, 2), dim3(WG), 0, st, p);
    return hipGetLastError();
}

}  // namespace ampd
