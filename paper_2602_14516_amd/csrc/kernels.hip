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
// fixed d; ds_read_b64_tr_b16 delivers exactly that from a row-major [key][d] tile.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace ampd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(uintptr_t)(p))

constexpr int WG = 256;
constexpr int KPAD = 16;     // bytes of padding per K row in LDS
constexpr int VPAD = 64;     // bytes of padding per V row in LDS
constexpr float NEG_INF = -__builtin_inff();

template <int D>
struct Geo {
    static constexpr int CPK = D / 8;                  // 16-byte (8-element) chunks per key row
    static constexpr int KSTR = D * 2 + KPAD;          // LDS row strides in bytes
    static constexpr int VSTR = D * 2 + VPAD;
    static constexpr int K32 = 32 * KSTR;              // bytes of a 32-key K block
    static constexpr int V32 = 32 * VSTR;
    static constexpr int WIDE_STAGE = 2 * (K32 + V32); // one 64-key stage (K then V)
    static constexpr int SMEM = 2 * WIDE_STAGE;        // two stages == four wave-private 32-key blocks
    static constexpr int NDB = D / 32;                 // 32-row blocks of O^T
    static constexpr int NKK = D / 16;                 // MFMA k-steps of the first product
};

// ---------------------------------------------------------------------------------------------
// small helpers

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

// 8 stored elements -> 8 bf16 (as a 16-byte vector) for LDS.
template <int KVT>
struct RawChunk;
template <>
struct RawChunk<KV_BF16> {
    u32x4 v;
    __device__ __forceinline__ void zero() { v = u32x4{0, 0, 0, 0}; }
    static constexpr int ES = 2;                      // bytes per stored element
    __device__ __forceinline__ void load(const char* base, uint32_t lane_off) {
        v = *reinterpret_cast<const u32x4*>(base + lane_off);
    }
    __device__ __forceinline__ u32x4 widen(float) const { return v; }
};
template <>
struct RawChunk<KV_FP8> {
    u32x2 v;
    __device__ __forceinline__ void zero() { v = u32x2{0, 0}; }
    static constexpr int ES = 1;
    __device__ __forceinline__ void load(const char* base, uint32_t lane_off) {
        v = *reinterpret_cast<const u32x2*>(base + lane_off);
    }
    // decode(code) * scale is exact in bf16: 4 significant bits times a power of two
    __device__ __forceinline__ u32x4 widen(float scale) const {
        uint32_t w[2] = {v.x, v.y};
        uint32_t o[4];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(w[h], false);
            f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(w[h], true);
            bf16x2 a = {(__bf16)(lo.x * scale), (__bf16)(lo.y * scale)};
            bf16x2 b = {(__bf16)(hi.x * scale), (__bf16)(hi.y * scale)};
            o[2 * h] = __builtin_bit_cast(uint32_t, a);
            o[2 * h + 1] = __builtin_bit_cast(uint32_t, b);
        }
        return u32x4{o[0], o[1], o[2], o[3]};
    }
};

struct ItemCtx {
    int req, kvh, g0, gn, q0, nq, kv_begin, kv_end, part_off;
    int C, L, row_off;
    const int32_t* bt_row;     // block-table row of the request
};

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
    const ReqInfo ri = p.reqs[it.req];
    c.C = ri.C;
    c.L = ri.L;
    c.row_off = ri.row_off;
    c.bt_row = p.block_table + (int64_t)it.req * p.max_pages;
    return c;
}

// Per-lane state of one wave: 32 query rows (lane % 32), O^T as D/32 accumulator blocks.
template <int D>
struct WaveAcc {
    f32x16 O[Geo<D>::NDB];
    float m;      // running max in the log2 domain (scale * log2(e) folded in)
    float l;      // this lane's share of the running sum (lanes l and l^32 hold halves)
};

// NB consecutive 32-key blocks: S^T = K Q^T, online softmax, O^T += V^T P^T.
//   kl / vl:  LDS addresses (bytes) of the first block's K and V rows; block j follows at
//             kl + j*kstep / vl + j*vstep
//   rel:      per lane, (last visible key of this lane's query) - (first key of block 0) - 4*(lane/32)
//   mask_from: first block index that needs the causal select (NB: none); wave-uniform
// The running maximum is a *reference* m, not the exact maximum: it is raised (and O, l
// rescaled) only when some row's block maximum exceeds it by more than RESCALE_SLACK in the
// log2 domain, so that probabilities stay below 2^RESCALE_SLACK.  (m, l, O) remain a
// consistent triple, which is all the final normalisation and the split-KV merge need.
constexpr float RESCALE_SLACK = 8.0f;

template <int D, int NB>
__device__ __forceinline__ void blocks(uint32_t kl, uint32_t vl, int kstep, int vstep,
                                       const bf16x8 (&Q)[Geo<D>::NKK], WaveAcc<D>& st, float c, int rel,
                                       int mask_from, int lane) {
    using G_ = Geo<D>;
    const int g = lane >> 5;
    f32x16 S[NB];
    const uint32_t ka = kl + (lane & 31) * G_::KSTR + g * 16;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        S[j] = f32x16{0};
#pragma unroll
        for (int kk = 0; kk < G_::NKK; ++kk) {
            const u32x4 raw = *LDS_PTR(const u32x4, ka + j * kstep + kk * 32);
            S[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), Q[kk], S[j], 0, 0, 0);
        }
    }
    if (mask_from < NB) {                              // wave-uniform: only blocks crossing the diagonal
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            if (j >= mask_from) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int koff = j * 32 + (i >> 2) * 8 + (i & 3);
                    S[j][i] = koff <= rel ? S[j][i] : NEG_INF;
                }
            }
        }
    }
    float mx = S[0][0];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int i = (j == 0 ? 1 : 0); i < 16; ++i) mx = fmaxf(mx, S[j][i]);
    mx = fmaxf(mx, xor32(mx)) * c;
    if (__any(mx > st.m + RESCALE_SLACK)) {            // rare after the first blocks
        const float m_new = fmaxf(st.m, mx);
        const float alpha = fast_exp2(st.m - (m_new == NEG_INF ? 0.0f : m_new));
        st.l *= alpha;
#pragma unroll
        for (int db = 0; db < G_::NDB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) st.O[db][i] *= alpha;
        st.m = m_new;
    }
    const float m_use = st.m == NEG_INF ? 0.0f : st.m;
    float psum = 0.0f;
    bf16x8 Pb[NB][2];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float pv = fast_exp2(__builtin_fmaf(S[j][i], c, -m_use));
            psum += pv;
            Pb[j][i >> 3][i & 7] = (__bf16)pv;
        }
    st.l += psum;
    // second product: k-slot s of MFMA cc is key 16*cc + 8*(s/4) + 4*g + s%4 of its block
    const int hi = (lane >> 4) & 1, i16 = lane & 15;
    const uint32_t va = vl + (4 * g + (i16 >> 2)) * G_::VSTR + (hi * 16 + (i16 & 3) * 4) * 2;
    typedef short s16x8 __attribute__((ext_vector_type(8)));
#pragma unroll
    for (int j = 0; j < NB; ++j) {
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
#pragma unroll
            for (int db = 0; db < G_::NDB; ++db) {
                const uint32_t a0 = va + j * vstep + (16 * cc) * G_::VSTR + db * 64;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0));
                const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0 + 8 * G_::VSTR));
                const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi4[0], hi4[1], hi4[2], hi4[3]};
                st.O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), Pb[j][cc], st.O[db], 0, 0, 0);
            }
        }
    }
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

// Cooperative K/V tile loader: NTHR threads move NKEYS consecutive keys (K and V rows) from the
// paged pools into registers and then into LDS.  Page ids are fetched one tile earlier than
// the K/V rows they address, so that the dependent block-table -> pool load chain is never on
// the critical path.  Within one pass a wave reads 64/CPK consecutive keys of one page, so
// the page id is wave-uniform: it is moved to a scalar register and the 64-bit address
// arithmetic runs on the scalar unit; the per-lane part of the address is a constant.
template <int D, int KVT, int NTHR, int NKEYS>
struct Loader {
    static constexpr int CPK = D / 8;                 // 8-element chunks per key row
    static constexpr int KPP = NTHR / CPK;            // keys per pass
    static constexpr int NPASS = NKEYS / KPP;
    static constexpr int KPW = 64 / CPK;              // keys per wave per pass
    static constexpr int ES = RawChunk<KVT>::ES;
    int pg[NPASS];
    RawChunk<KVT> k[NPASS], v[NPASS];
    float ks[NPASS], vs[NPASS];

    // t: thread index inside the group of NTHR threads
    __device__ __forceinline__ void fetch_pages(const AttnParams& p, const ItemCtx& ic, int kbase, int t) {
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int key0 = kbase + ps * KPP + (t >> 6) * KPW;
            pg[ps] = key0 < ic.kv_end ? ic.bt_row[key0 >> p.logP] : 0;
        }
    }

    template <bool FULL>
    __device__ __forceinline__ void fetch_kv_impl(const AttnParams& p, const ItemCtx& ic, int kbase, int t) {
        const uint32_t lane_off = (uint32_t)(((t & 63) / CPK) * D + (t % CPK) * 8) * ES;
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int key0 = __builtin_amdgcn_readfirstlane(kbase + ps * KPP + (t >> 6) * KPW);
            const int page = __builtin_amdgcn_readfirstlane(pg[ps]);
            const int64_t row = ((((int64_t)page * p.Hkv + ic.kvh) << p.logP) + (key0 & (p.P - 1))) * D * ES;
            const char* kb = static_cast<const char*>(p.k_pool) + row;
            const char* vb = static_cast<const char*>(p.v_pool) + row;
            ks[ps] = 1.0f;
            vs[ps] = 1.0f;
            if (KVT == KV_FP8) {
                ks[ps] = p.k_scale[(int64_t)page * p.Hkv + ic.kvh];
                vs[ps] = p.v_scale[(int64_t)page * p.Hkv + ic.kvh];
            }
            if (FULL || key0 + (t & 63) / CPK < ic.kv_end) {
                k[ps].load(kb, lane_off);
                v[ps].load(vb, lane_off);
            } else {
                k[ps].zero();                                    // keys past the item's end: zeros, so
                v[ps].zero();                                    // that 0-weights never meet NaN garbage
            }
        }
    }

    __device__ __forceinline__ void fetch_kv(const AttnParams& p, const ItemCtx& ic, int kbase, int t) {
        if (kbase + NKEYS <= ic.kv_end)                          // uniform: whole tile inside the key range
            fetch_kv_impl<true>(p, ic, kbase, t);
        else
            fetch_kv_impl<false>(p, ic, kbase, t);
    }

    // kl / vl: LDS byte addresses of key 0 of this tile's K and V rows
    __device__ __forceinline__ void commit(uint32_t kl, uint32_t vl, int t) const {
        const int ch = t % CPK;
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int kloc = ps * KPP + t / CPK;
            *LDS_PTR(u32x4, kl + kloc * Geo<D>::KSTR + ch * 16) = k[ps].widen(ks[ps]);
            *LDS_PTR(u32x4, vl + kloc * Geo<D>::VSTR + ch * 16) = v[ps].widen(vs[ps]);
        }
    }
};

// Final write of one wave's O^T: either bf16 output rows or fp32 partials.
//   row_in_item: this lane's row index inside the item (token_local * gn + head) or -1
template <int D>
__device__ __forceinline__ void store_result(const AttnParams& p, const ItemCtx& ic, WaveAcc<D>& st,
                                             int tok, int head_in_group, int row_in_item, int lane) {
    using G_ = Geo<D>;
    const int g = lane >> 5;
    const float ltot = st.l + xor32(st.l);
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
// wide body: 4 waves x 32 query rows share 64-key K/V tiles, double-buffered in LDS

template <int D, int KVT>
__device__ __forceinline__ void wide_body(const AttnParams& p, const ItemCtx& ic, uint32_t smem) {
    using G_ = Geo<D>;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tqw = 32 / ic.gn;                            // tokens per wave
    const int row = lane & 31;
    const int tl = row / ic.gn, hg = row - tl * ic.gn;
    const int tok_local = wave * tqw + tl;                 // token index inside the item
    const bool valid = tl < tqw && tok_local < ic.nq;
    const int tok = ic.q0 + tok_local;
    // wave-level causal bounds (last visible key = C + token)
    const int w_first = ic.C + ic.q0 + wave * tqw;
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
    const int ntiles = (ic.kv_end - k_lo + 63) >> 6;
    Loader<D, KVT, WG, 64> ld;
    ld.fetch_pages(p, ic, k_lo, tid);
    ld.fetch_kv(p, ic, k_lo, tid);
    if (ntiles > 1) ld.fetch_pages(p, ic, k_lo + 64, tid);
    ld.commit(smem, smem + 2 * G_::K32, tid);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const uint32_t cur = smem + (t & 1) * G_::WIDE_STAGE;
        const uint32_t nxt = smem + ((t + 1) & 1) * G_::WIDE_STAGE;
        const bool more = t + 1 < ntiles;
        if (more) {
            ld.fetch_kv(p, ic, k_lo + (t + 1) * 64, tid);
            if (t + 2 < ntiles) ld.fetch_pages(p, ic, k_lo + (t + 2) * 64, tid);
        }
        const int kbase = k_lo + t * 64;
        if (wave_active && kbase <= w_last) {               // else every row of the wave masks this tile
            const int rel = lim - kbase - 4 * (lane >> 5);
            // block j (32 keys) needs the causal select iff its last key is beyond the wave's first limit
            const int mask_from = kbase + 31 > w_first ? 0 : (kbase + 63 > w_first ? 1 : 2);
            blocks<D, 2>(cur, cur + 2 * G_::K32, G_::K32, G_::V32, Q, st, p.c_log2, rel, mask_from, lane);
        }
        if (more) ld.commit(nxt, nxt + 2 * G_::K32, tid);
        __syncthreads();
    }
    store_result<D>(p, ic, st, tok, hg, valid ? tok_local * ic.gn + hg : -1, lane);
}

// ---------------------------------------------------------------------------------------------
// narrow body: <= 32 query rows; the 4 waves take 32-key blocks round-robin, each through its
// own LDS region, and merge their (m, l, O) through LDS at the end

template <int D, int KVT>
__device__ __forceinline__ void narrow_body(const AttnParams& p, const ItemCtx& ic, uint32_t smem) {
    using G_ = Geo<D>;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = lane & 31;
    const int tl = row / ic.gn, hg = row - tl * ic.gn;
    const bool valid = tl < ic.nq;
    const int tok = ic.q0 + tl;
    const int lim = valid ? ic.C + tok : 0x3fffffff;
    const int first_lim = ic.C + ic.q0;                  // smallest last-visible key among the rows

    bf16x8 Q[G_::NKK];
    load_q<D>(p, ic, tok, hg, valid, lane, Q);
    WaveAcc<D> st;
#pragma unroll
    for (int db = 0; db < G_::NDB; ++db) st.O[db] = f32x16{0};
    st.m = NEG_INF;
    st.l = 0.0f;

    const uint32_t kl = smem + wave * (G_::K32 + G_::V32);
    const uint32_t vl = kl + G_::K32;
    const int nblocks = (ic.kv_end - ic.kv_begin + 31) >> 5;
    Loader<D, KVT, 64, 32> ld;
    if (wave < nblocks) {
        ld.fetch_pages(p, ic, ic.kv_begin + wave * 32, lane);
        ld.fetch_kv(p, ic, ic.kv_begin + wave * 32, lane);
        if (wave + 4 < nblocks) ld.fetch_pages(p, ic, ic.kv_begin + (wave + 4) * 32, lane);
    }
    for (int b = wave; b < nblocks; b += 4) {
        const int kbase = ic.kv_begin + b * 32;
        ld.commit(kl, vl, lane);
        if (b + 4 < nblocks) {
            ld.fetch_kv(p, ic, kbase + 128, lane);
            if (b + 8 < nblocks) ld.fetch_pages(p, ic, kbase + 256, lane);
        }
        const int rel = lim - kbase - 4 * (lane >> 5);
        blocks<D, 1>(kl, vl, 0, 0, Q, st, p.c_log2, rel, kbase + 31 > first_lim ? 0 : 1, lane);
    }
    // merge the four waves: LDS holds O as [wave][row 0..31][D + 4] fp32 and (m, l) as [wave][32][2]
    const float ltot = st.l + xor32(st.l);
    __syncthreads();                                      // every wave is done with its K/V region
    constexpr int OSTR = D + 4;
    const uint32_t obase = smem;
    const uint32_t mlbase = smem + 4 * 32 * OSTR * 4;
    {
        const int g = lane >> 5;
        const uint32_t orow = obase + ((wave * 32 + row) * OSTR) * 4;
#pragma unroll
        for (int db = 0; db < G_::NDB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int d0 = db * 32 + i4 * 8 + g * 4;
                f32x4 o = {st.O[db][i4 * 4], st.O[db][i4 * 4 + 1], st.O[db][i4 * 4 + 2], st.O[db][i4 * 4 + 3]};
                *LDS_PTR(f32x4, orow + d0 * 4) = o;
            }
        if (g == 0) {
            *LDS_PTR(float, mlbase + ((wave * 32 + row) * 2) * 4) = st.m;
            *LDS_PTR(float, mlbase + ((wave * 32 + row) * 2 + 1) * 4) = ltot;
        }
    }
    __syncthreads();
    // thread -> (row r, 16 consecutive d) for D = 128; (row, 8 d) for D = 64
    constexpr int DPT = D / 8;
    const int r = tid >> 3, dc = (tid & 7) * DPT;
    const int rows = ic.nq * ic.gn;
    if (r < rows) {
        float mw[4], lw[4];
        float mall = NEG_INF;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            mw[w] = *LDS_PTR(float, mlbase + ((w * 32 + r) * 2) * 4);
            lw[w] = *LDS_PTR(float, mlbase + ((w * 32 + r) * 2 + 1) * 4);
            mall = fmaxf(mall, mw[w]);
        }
        const float muse = mall == NEG_INF ? 0.0f : mall;
        float lsum = 0.0f, wgt[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            wgt[w] = fast_exp2(mw[w] - muse);
            lsum += lw[w] * wgt[w];
        }
        float acc[DPT];
#pragma unroll
        for (int x = 0; x < DPT; ++x) acc[x] = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
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
            for (int x = 0; x < DPT; x += 8) {
                bf16x8 o;
#pragma unroll
                for (int y = 0; y < 8; ++y) o[y] = (__bf16)(acc[x + y] * inv);
                *reinterpret_cast<u32x4*>(dst + x * 2) = __builtin_bit_cast(u32x4, o);
            }
        } else {
            float* po = p.partial + ic.part_off + (int64_t)r * D + dc;
#pragma unroll
            for (int x = 0; x < DPT; x += 4) {
                f32x4 o = {acc[x], acc[x + 1], acc[x + 2], acc[x + 3]};
                *reinterpret_cast<f32x4*>(po + x) = o;
            }
            if ((tid & 7) == 0) {
                float* ml = p.partial + ic.part_off + (int64_t)rows * D + r * 2;
                ml[0] = mall;
                ml[1] = lsum;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// the fused attention launch: one workgroup per work item, wide and narrow items in one grid

template <int D, int KVT>
__global__ __launch_bounds__(WG, 2) void attn_kernel(const AttnParams p) {
    __shared__ __attribute__((aligned(16))) char smem_raw[Geo<D>::SMEM];
    const uint32_t smem = (uint32_t)(uintptr_t)LDS_PTR(char, smem_raw);
    const ItemCtx ic = load_item(p, blockIdx.x);
    const int kind = (p.items[blockIdx.x].heads >> 24) & 0xff;
    if (kind == KIND_WIDE)
        wide_body<D, KVT>(p, ic, smem);
    else
        narrow_body<D, KVT>(p, ic, smem);
}

// ---------------------------------------------------------------------------------------------
// combine: merge the split-KV partials of one query tile
//   m = max_s m_s;  l = sum_s l_s 2^(m_s - m);  O = sum_s O_s 2^(m_s - m) / l

template <int D>
__global__ __launch_bounds__(WG) void combine_kernel(const AttnParams p) {
    const CombItem ci = p.combs[blockIdx.x];
    const int kvh = ci.heads & 0xff, g0 = (ci.heads >> 8) & 0xff, gn = (ci.heads >> 16) & 0xff;
    const ReqInfo ri = p.reqs[ci.req];
    const int rows = ci.nq * gn;
    constexpr int QPR = D / 4;                         // float4 groups per row
    for (int u = threadIdx.x; u < rows * QPR; u += WG) {
        const int r = u / QPR, dq = (u % QPR) * 4;
        float mall = NEG_INF;
        for (int s = 0; s < ci.nsplit; ++s) {
            const float* ml = p.partial + ci.part_off + (int64_t)s * ci.part_stride + (int64_t)rows * D + r * 2;
            mall = fmaxf(mall, ml[0]);
        }
        const float muse = mall == NEG_INF ? 0.0f : mall;
        float lsum = 0.0f;
        f32x4 acc = {0, 0, 0, 0};
        for (int s = 0; s < ci.nsplit; ++s) {
            const float* base = p.partial + ci.part_off + (int64_t)s * ci.part_stride;
            const float* ml = base + (int64_t)rows * D + r * 2;
            const float w = fast_exp2(ml[0] - muse);
            lsum += ml[1] * w;
            const f32x4 o = *reinterpret_cast<const f32x4*>(base + (int64_t)r * D + dq);
            acc += o * w;
        }
        const float inv = 1.0f / lsum;
        const int tl = r / gn, hg = r - tl * gn;
        const int hq = kvh * (p.Hq / p.Hkv) + g0 + hg;
        char* dst = static_cast<char*>(p.out) + (((int64_t)(ri.row_off + ci.q0 + tl) * p.Hq + hq) * D + dq) * 2;
        bf16x4 o = {(__bf16)(acc[0] * inv), (__bf16)(acc[1] * inv), (__bf16)(acc[2] * inv), (__bf16)(acc[3] * inv)};
        *reinterpret_cast<u32x2*>(dst) = __builtin_bit_cast(u32x2, o);
    }
}

// ---------------------------------------------------------------------------------------------
// KV append, bf16 cache: a bit-exact scatter.  grid = (pages touched, requests, 2 {K,V})

__global__ __launch_bounds__(WG) void append_bf16_kernel(const AppendParams p) {
    const int r = blockIdx.y;
    const int C = p.C[r], L = p.L[r];
    const int lp = (C >> p.logP) + blockIdx.x;               // logical page
    const int t0 = max(C, lp << p.logP), t1 = min(C + L, (lp + 1) << p.logP);
    if (t0 >= t1) return;
    const int page = p.block_table[(int64_t)(p.req0 + r) * p.max_pages + lp];
    const int cpt = p.Hkv * p.D / 8;                         // 16-byte chunks per token
    const int cph = p.D / 8;
    const char* src = static_cast<const char*>(blockIdx.z ? p.v_new : p.k_new);
    char* dst = static_cast<char*>(blockIdx.z ? p.v_pool : p.k_pool);
    const int total = (t1 - t0) * cpt;
    for (int u = threadIdx.x; u < total; u += WG) {
        const int t = t0 + u / cpt, rem = u % cpt;
        const int h = rem / cph, ch = rem % cph;
        const u32x4 v = *reinterpret_cast<const u32x4*>(src + (((int64_t)(p.row_off[r] + t - C) * p.Hkv + h) * p.D + ch * 8) * 2);
        const int64_t e = ((((int64_t)page * p.Hkv + h) << p.logP) + (t & (p.P - 1))) * p.D + ch * 8;
        *reinterpret_cast<u32x4*>(dst + e * 2) = v;
    }
}

// KV append, 8-bit cache.  grid = (pages touched, requests, 2 {K,V}); the block walks the KV
// heads; per head: amax of the new tokens -> exponent -> (re-encode old slots) -> encode.
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
    const int r = blockIdx.y;
    const int C = p.C[r], L = p.L[r];
    const int lp = (C >> p.logP) + blockIdx.x;
    const int t0 = max(C, lp << p.logP), t1 = min(C + L, (lp + 1) << p.logP);
    if (t0 >= t1) return;
    const int page = p.block_table[(int64_t)(p.req0 + r) * p.max_pages + lp];
    const int n_old = max(0, C - (lp << p.logP));
    const char* src = static_cast<const char*>(blockIdx.z ? p.v_new : p.k_new);
    uint8_t* dst = static_cast<uint8_t*>(blockIdx.z ? p.v_pool : p.k_pool);
    float* scl = blockIdx.z ? p.v_scale : p.k_scale;
    const int cph = p.D / 8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int h = 0; h < p.Hkv; ++h) {
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
        __syncthreads();                                       // red / e_sh are reused by the next head
    }
}

// ---------------------------------------------------------------------------------------------
// launchers

template <int D, int KVT>
static hipError_t launch_attn_t(const AttnParams& p, int nitems, hipStream_t st) {
    hipLaunchKernelGGL((attn_kernel<D, KVT>), dim3(nitems), dim3(WG), 0, st, p);
    return hipGetLastError();
}

hipError_t launch_attn(const AttnParams& p, int D, int kvt, int nitems, hipStream_t st) {
    if (nitems <= 0) return hipSuccess;
    if (D == 128 && kvt == KV_BF16) return launch_attn_t<128, KV_BF16>(p, nitems, st);
    if (D == 64 && kvt == KV_BF16) return launch_attn_t<64, KV_BF16>(p, nitems, st);
    if (D == 128 && kvt == KV_FP8) return launch_attn_t<128, KV_FP8>(p, nitems, st);
    if (D == 64 && kvt == KV_FP8) return launch_attn_t<64, KV_FP8>(p, nitems, st);
    return hipErrorInvalidValue;
}

hipError_t launch_combine(const AttnParams& p, int D, int ncombs, hipStream_t st) {
    if (ncombs <= 0) return hipSuccess;
    if (D == 128)
        hipLaunchKernelGGL((combine_kernel<128>), dim3(ncombs), dim3(WG), 0, st, p);
    else
        hipLaunchKernelGGL((combine_kernel<64>), dim3(ncombs), dim3(WG), 0, st, p);
    return hipGetLastError();
}

hipError_t launch_append(const AppendParams& p, int kvt, int max_pages_touched, int nreq, hipStream_t st) {
    if (nreq <= 0 || max_pages_touched <= 0) return hipSuccess;
    if (kvt == KV_BF16)
        hipLaunchKernelGGL(append_bf16_kernel, dim3(max_pages_touched, nreq, 2), dim3(WG), 0, st, p);
    else
        hipLaunchKernelGGL(append_fp8_kernel, dim3(max_pages_touched, nreq, 2), dim3(WG), 0, st, p);
    return hipGetLastError();
}

}  // namespace ampd
