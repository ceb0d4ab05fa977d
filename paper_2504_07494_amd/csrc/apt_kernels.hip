// HIP kernels (gfx950) of the hybrid-cache decode attention step and their launchers.
//
//   items kernel   one workgroup (4 wavefronts of 64) per work item of the plan:
//                    KV-kind item      streams the K and V rows of one head over a token
//                                      range, online softmax per 16-lane group (HBM bound)
//                    hidden-kind item  projects K_h, V_h of a 256-token tile from the
//                                      gathered hidden rows on MFMA (or on plain ALUs
//                                      for fp32) and attends to them from registers
//                  every item writes one partial (m, l, acc[head_dim]) in fp32
//   merge kernel   combines a request's partials per head and normalises
//   apt_absorbed.inc: the hidden-kind requests without the projection (opt-in, APT_HIDDEN_ABSORBED)
//   cache append / cache write, weight packing, calibration kernels
//
// Scores are kept in base-2 units: s2 = softmax_scale*log2(e)*<q,k>, weights 2^(s2 - m).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <mutex>
#include "apt_internal.h"
#include "apt_hybrid_bench.h"

// Workspace of apt_hybrid_decode_attn_static: one copy per device, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; the device address is looked up once per device (device_setup).
static __device__ __align__(256) unsigned char scratch[APT_STATIC_WORKSPACE_BYTES];

namespace {

constexpr float kSentinel = -1.0e30f;   // "no score yet": finite, so differences never give NaN
constexpr int kThreads = 256;

typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// 16-byte load of data that is read once (streamed past the caches)
__device__ inline uint4 load16_stream(const char* p) {
    const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

struct ItemParams {
    const int32_t* plan;          // device blob
    int32_t* kv_ticket;           // device blob word APT_PW_KV_TICKET: next KV-kind item of the persistent launch
    const char* q;
    const char* k_pages;
    const char* v_pages;
    const char* hidden_pages;
    const char* W_K;
    const char* W_V;
    const char* W_packed;
    const char* b_K;
    const char* b_V;
    const int32_t* block_tables;
    float* ws_acc;                // [n_slots][HD]
    float2* ws_ml;                // [n_slots]
    int32_t B, H, d, bs, log2_bs, max_blocks;
    int32_t n_items, n_hidden_items, hidden_chunk, kv_chunk, items_off;
    float scale_log2e;
    int32_t item_base;            // one-workgroup-per-item launch: first item of the grid
    // absorbed-weight hidden path: workspace sections (fp32)
    float* ab_qt;                 // [n_hid_req][H][d]
    float* ab_cb;                 // [n_hid_req][H]
    float* ab_s;                  // [KS][H][ab_tokens] partial scores over d_model slices; slice 0 ends as the scores
    float2* ab_ml;                // [n_hid_req][H]
    float* ab_yp;                 // [n_hidden_items][H][d]
    float* ab_op;                 // [KS][n_hid_req][H][HD]
    void* ab_pp;                  // 16-bit inputs: softmax weights as 16-bit parts, [16 n_hidden_items][parts * 64][32]
    int64_t ab_tokens;            // cached tokens of all hidden-kind requests
    int32_t n_hid_req;
};

// ---------------------------------------------------------------------------------
// element helpers.  DT: 0 = fp32, 1 = fp16, 2 = bf16
// ---------------------------------------------------------------------------------
template <int DT> struct Elt { static constexpr int bytes = DT == 0 ? 4 : 2; static constexpr int per16 = 16 / bytes; };

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

template <int DT> __device__ inline float load_elem(const char* base, int64_t idx) {
    if constexpr (DT == 0) return ((const float*)base)[idx];
    else if constexpr (DT == 1) return (float)((const _Float16*)base)[idx];
    else return bf16_to_f32(((const uint16_t*)base)[idx]);
}

// 16 bytes -> Elt<DT>::per16 floats
template <int DT> __device__ inline void cvt16(const uint4& v, float* out) {
    if constexpr (DT == 0) {
        out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y);
        out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
    } else if constexpr (DT == 1) {
        h8_t h = __builtin_bit_cast(h8_t, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = (float)h[i];
    } else {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
}

__device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---------------------------------------------------------------------------------
// cross-lane helpers
// ---------------------------------------------------------------------------------
template <int CTRL> __device__ inline float dpp_mov(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
// Sum over the aligned group of LANES lanes a lane belongs to; every lane gets the sum.
template <int LANES> __device__ inline float group_sum(float x) {
    x += dpp_mov<0xB1>(x);                          // quad_perm [1,0,3,2]
    x += dpp_mov<0x4E>(x);                          // quad_perm [2,3,0,1]
    if constexpr (LANES >= 8) x += dpp_mov<0x141>(x);   // row_half_mirror
    if constexpr (LANES >= 16) x += dpp_mov<0x140>(x);  // row_mirror
    if constexpr (LANES >= 32) x += __shfl_xor(x, 16);
    if constexpr (LANES >= 64) x += __shfl_xor(x, 32);
    return x;
}
template <int LANES> __device__ inline float group_max(float x) {
    x = fmaxf(x, dpp_mov<0xB1>(x));
    x = fmaxf(x, dpp_mov<0x4E>(x));
    if constexpr (LANES >= 8) x = fmaxf(x, dpp_mov<0x141>(x));
    if constexpr (LANES >= 16) x = fmaxf(x, dpp_mov<0x140>(x));
    if constexpr (LANES >= 32) x = fmaxf(x, __shfl_xor(x, 16));
    if constexpr (LANES >= 64) x = fmaxf(x, __shfl_xor(x, 32));
    return x;
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---------------------------------------------------------------------------------
// KV-kind item
// ---------------------------------------------------------------------------------
// K/V block layout [head][slot][HD]: the rows of one (block, head) are one contiguous run
// of bs*HD elements, read as 1 KB wave loads (64 lanes x 16 B).  LPR lanes share a row,
// 64/LPR rows per load.  A lane group keeps its own online-softmax state for the rows it
// sees; the groups are combined through LDS at the end.
constexpr int kKvUnits = 4;   // 1 KB loads of K (and of V) per pipeline stage

template <int DT, int HD>
__device__ __forceinline__ void kv_item(const ItemParams& p, int r, int h, int t0, int t1, char* lds) {
    constexpr int EB = Elt<DT>::bytes;
    constexpr int EPL = Elt<DT>::per16;          // elements per lane per load
    constexpr int LPR = HD * EB / 16;            // lanes per row
    constexpr int RPL = 64 / LPR;                // rows per 1 KB load
    constexpr int G = 4 * RPL;                   // lane groups in the workgroup

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int bs = p.bs;
    const int log2_nl = p.log2_bs - __builtin_ctz(RPL);     // loads per page per matrix = bs/RPL
    const int nl_mask = (1 << log2_nl) - 1;
    const int64_t blk_bytes = (int64_t)bs * p.d * EB;
    const int64_t head_off = (int64_t)h * bs * HD * EB;

    const int p0 = t0 >> p.log2_bs;
    const int p1 = (t1 + bs - 1) >> p.log2_bs;
    // pages of this wave: p0 + w, p0 + w + 4, ...
    const int npg = (p1 - p0 - w + 3) >> 2;
    const int nunits = npg > 0 ? (npg << log2_nl) : 0;

    // lane i holds the block ids of the wave's i-th page
    int32_t kid = 0, vid = 0;
    if (lane < npg) {
        const int64_t e = (int64_t)r * 2 * p.max_blocks + p0 + w + 4 * lane;
        kid = p.block_tables[e];
        vid = p.block_tables[e + p.max_blocks];
    }

    // q for the lane's channels, pre-scaled
    const int c0 = (lane % LPR) * EPL;
    float qf[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i)
        qf[i] = load_elem<DT>(p.q, ((int64_t)r * p.H + h) * HD + c0 + i) * p.scale_log2e;

    float m = kSentinel, l = 0.f, acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;

    uint4 kb[2][kKvUnits], vb[2][kKvUnits];
    auto issue = [&](int g, uint4* kbuf, uint4* vbuf) {
#pragma unroll
        for (int i = 0; i < kKvUnits; ++i) {
            const int u = g * kKvUnits + i;
            if (u < nunits) {
                const int pg = u >> log2_nl;
                const int64_t kblk = __builtin_amdgcn_readlane(kid, pg);
                const int64_t vblk = __builtin_amdgcn_readlane(vid, pg);
                const int64_t off = head_off + (int64_t)(u & nl_mask) * 1024 + lane * 16;
                kbuf[i] = load16_stream(p.k_pages + kblk * blk_bytes + off);
                vbuf[i] = load16_stream(p.v_pages + vblk * blk_bytes + off);
            }
        }
    };
    auto consume = [&](int g, const uint4* kbuf, const uint4* vbuf) {
        float s[kKvUnits];
        bool ok[kKvUnits];
        float mn = m;
#pragma unroll
        for (int i = 0; i < kKvUnits; ++i) {
            const int u = g * kKvUnits + i;
            const int pg = u >> log2_nl;
            const int tok = ((p0 + w + 4 * pg) << p.log2_bs) + (u & nl_mask) * RPL + lane / LPR;
            ok[i] = (u < nunits) && (tok < t1);
            float kf[EPL];
            cvt16<DT>(kbuf[i], kf);
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) part = fmaf(kf[e], qf[e], part);
            part = group_sum<LPR>(part);
            s[i] = ok[i] ? part : kSentinel;
            mn = fmaxf(mn, s[i]);
        }
        const float alpha = fast_exp2(m - mn);
        l *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
#pragma unroll
        for (int i = 0; i < kKvUnits; ++i) {
            const float pw = ok[i] ? fast_exp2(s[i] - mn) : 0.f;
            l += pw;
            float vf[EPL];
            cvt16<DT>(vbuf[i], vf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(pw, ok[i] ? vf[e] : 0.f, acc[e]);
        }
        m = mn;
    };

    const int ngroups = (nunits + kKvUnits - 1) / kKvUnits;
    if (ngroups > 0) issue(0, kb[0], vb[0]);
    for (int g = 0; g < ngroups; g += 2) {
        if (g + 1 < ngroups) issue(g + 1, kb[1], vb[1]);
        consume(g, kb[0], vb[0]);
        if (g + 2 < ngroups) issue(g + 2, kb[0], vb[0]);
        if (g + 1 < ngroups) consume(g + 1, kb[1], vb[1]);
    }

    // combine the lane groups: LDS [G] m, [G] l, [G][HD] acc
    float* gm = (float*)lds;
    float* gl = gm + G;
    float* ga = gl + G;
    const int grp = w * RPL + lane / LPR;
    if (lane % LPR == 0) { gm[grp] = m; gl[grp] = l; }
#pragma unroll
    for (int e = 0; e < EPL; ++e) ga[grp * HD + c0 + e] = acc[e];
    __syncthreads();
    if (tid < HD) {
        float M = kSentinel;
        for (int g = 0; g < G; ++g) M = fmaxf(M, gm[g]);
        float L = 0.f, A = 0.f;
        for (int g = 0; g < G; ++g) {
            const float wgt = fast_exp2(gm[g] - M);
            L = fmaf(gl[g], wgt, L);
            A = fmaf(ga[g * HD + tid], wgt, A);
        }
        const int32_t* split_count = p.plan + APT_PW_HEADER;
        const int32_t* ws_offset = split_count + p.B;
        const int64_t slot = ((int64_t)ws_offset[r] + t0 / p.kv_chunk) * p.H + h;
        p.ws_acc[slot * HD + tid] = A;
        if (tid == 0) p.ws_ml[slot] = make_float2(M, L);
    }
}

// ---------------------------------------------------------------------------------
// hidden-kind item, plain-ALU version (fp32 configs and shapes the MFMA kernel
// does not cover).  chunk <= 64 tokens.
// ---------------------------------------------------------------------------------
template <int DT, int HD>
__device__ __forceinline__ void hidden_item_valu(const ItemParams& p, int r, int h, int t0, int t1, char* lds) {
    constexpr int NG = kThreads / HD;     // token groups
    constexpr int TJ = 4;                 // tokens per pass of a thread
    constexpr int LD = HD + 1;
    const int C = p.hidden_chunk;
    float* Ks = (float*)lds;              // [C][LD]
    float* Vs = Ks + C * LD;              // [C][LD]
    float* sc = Vs + C * LD;              // [64]
    float* red = sc + 64;                 // [2]
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int c = tid % HD, g = tid / HD;
    const int n = t1 - t0;
    const int d = p.d;
    const int64_t blk_elems = (int64_t)p.bs * d;

    const float bk = load_elem<DT>(p.b_K, (int64_t)h * HD + c);
    const float bv = load_elem<DT>(p.b_V, (int64_t)h * HD + c);
    for (int j0 = g * TJ; j0 < n; j0 += NG * TJ) {
        int64_t xoff[TJ];
#pragma unroll
        for (int t = 0; t < TJ; ++t) {
            int tok = t0 + j0 + t;
            tok = tok < t1 ? tok : t1 - 1;
            const int64_t blk = p.block_tables[(int64_t)r * 2 * p.max_blocks + (tok >> p.log2_bs)];
            xoff[t] = blk * blk_elems + (int64_t)(tok & (p.bs - 1)) * d;
        }
        float ak[TJ], av[TJ];
#pragma unroll
        for (int t = 0; t < TJ; ++t) { ak[t] = bk; av[t] = bv; }
        for (int i = 0; i < d; ++i) {
            const float wk = load_elem<DT>(p.W_K, (int64_t)i * d + (int64_t)h * HD + c);
            const float wv = load_elem<DT>(p.W_V, (int64_t)i * d + (int64_t)h * HD + c);
#pragma unroll
            for (int t = 0; t < TJ; ++t) {
                const float x = load_elem<DT>(p.hidden_pages, xoff[t] + i);
                ak[t] = fmaf(x, wk, ak[t]);
                av[t] = fmaf(x, wv, av[t]);
            }
        }
#pragma unroll
        for (int t = 0; t < TJ; ++t)
            if (j0 + t < n) { Ks[(j0 + t) * LD + c] = ak[t]; Vs[(j0 + t) * LD + c] = av[t]; }
    }
    __syncthreads();
    for (int j = tid; j < n; j += kThreads) {
        float s = 0.f;
        for (int cc = 0; cc < HD; ++cc)
            s = fmaf(Ks[j * LD + cc], load_elem<DT>(p.q, ((int64_t)r * p.H + h) * HD + cc), s);
        sc[j] = s * p.scale_log2e;
    }
    __syncthreads();
    if (w == 0) {
        const float v = lane < n ? sc[lane] : kSentinel;
        const float m = group_max<64>(v);
        const float pw = lane < n ? fast_exp2(v - m) : 0.f;
        const float l = group_sum<64>(pw);
        sc[lane] = pw;
        if (lane == 0) { red[0] = m; red[1] = l; }
    }
    __syncthreads();
    if (tid < HD) {
        float a = 0.f;
        for (int j = 0; j < n; ++j) a = fmaf(sc[j], Vs[j * LD + tid], a);
        const int32_t* split_count = p.plan + APT_PW_HEADER;
        const int32_t* ws_offset = split_count + p.B;
        const int64_t slot = ((int64_t)ws_offset[r] + t0 / p.hidden_chunk) * p.H + h;
        p.ws_acc[slot * HD + tid] = a;
        if (tid == 0) p.ws_ml[slot] = make_float2(red[0], red[1]);
    }
}

// ---------------------------------------------------------------------------------
// hidden-kind items, MFMA version (fp16 / bf16, head_dim 128): persistent workgroups
// ---------------------------------------------------------------------------------
// Per item: K_h and V_h of a tile of up to 320 tokens (TF = 10; described here) or 256 tokens (TF = 8),
// [256 channels] x [320 tokens] with k = d_model, on v_mfma_f32_16x16x32.  The four waves are (mat, th): mat 0 = K_h channels, mat 1 =
// V_h channels; th picks the token blocks 2b + th (b = 0..4, 32 tokens each), so a short tile leaves
// both halves the same number of blocks.  A wave owns a 128 x 160 accumulator tile as 8 x 10 MFMA
// tiles of 16 x 16: 320 registers, more than the 256 AGPRs, so part of it lives in ordinary VGPRs.
// The tile is as large as the register file allows because the kernel is bound by the L2 -> LDS
// copies as much as by the matrix pipes: per k-tile a workgroup copies (256 + 320) rows of 64 B for
// 256 x 320 x 32 multiply-adds, 10 % fewer bytes per flop than a 256 x 256 tile, and a k-tile lasts
// 25 % longer, which is that much more latency the four stages can cover.
// K waves multiply W (rows = channels) by X^T and get D[channel][token]: a lane owns one token per
// tile column and sums over channels in registers for the score.  V waves multiply X (rows =
// tokens) by W^T and get D[token][channel]: a lane owns one channel and sums over tokens in
// registers for the weighted value sum.  Both read the same LDS images; only which image feeds
// which MFMA operand differs.
//
// k runs in tiles of 32 (one MFMA k-step) through four LDS stages, each 16 KB of packed weights
// (already in LDS order in memory) and 20 KB of X rows, filled by global->LDS copies that bypass
// registers; up to four k-tiles are in flight or waiting while one is multiplied.  Rows are 64 B;
// the 16-byte unit c of a row sits at c ^ swz16(row), which keeps the row-wise copies and the
// column-wise operand reads spread over all banks.  The operands of k-tile kt+1 are read into a
// second register set while k-tile kt is multiplied.
//
// A workgroup walks a queue of items (queue = blockIdx % 8, the XCD the workgroup runs
// on, so that the workgroups sharing an L2 work on few heads and few token tiles at a
// time), then a share of the KV-kind items.  While one item's epilogue runs, the first
// k-tiles of the next item are already on their way into LDS.
constexpr int kBK = 32;
constexpr int kRowBytes = kBK * 2;                     // 64 B
constexpr int kWTileBytes = 256 * kRowBytes;           // 16 KB
constexpr int kStages = 4;
constexpr int kXImage = kStages * kWTileBytes;         // LDS offset of the X stages
constexpr int kMfmaScratch = 5120;                     // epilogue scratch behind the stages
constexpr int kFragBytes = 16 * kRowBytes;             // the 16 rows of one MFMA operand fragment
// TF = X fragments (16 tokens) per wave: 10 (tile of 320 tokens) or 8 (256 tokens)
template <int TF> struct MfmaTile {
    static constexpr int kTokTile = 32 * TF;                   // token rows of a tile
    static constexpr int kXChunks = kTokTile / 64;             // 1 KB copies of X rows per wave and k-tile
    static constexpr int kXTileBytes = kTokTile * kRowBytes;   // 20 KB / 16 KB
    static constexpr int kLds = kStages * (kWTileBytes + kXTileBytes) + kMfmaScratch;
    static constexpr int kStageLoads = 4 + kXChunks;           // copies per wave and k-tile: 4 of W, then those of X
    static_assert(kTokTile % 64 == 0 && kLds <= 160 * 1024 && (TF == 8 || TF == 10), "tile does not fit");
};

// Position swizzles of the 16-byte units of 64-byte LDS rows, measured free of bank conflicts (SQ_LDS_BANK_CONFLICT = 0,
// 4 cycles per ds_read_b128) for the operand reads of the two MFMA forms: swz for 32x32x16 (a read covers 32 consecutive
// rows, two units; used by the absorbed-weight kernels), swz16 for 16x16x32 (16 consecutive rows, all four units; with
// swz it takes 8 cycles).
__host__ __device__ inline int swz(int row) { return (row >> 2) & 3; }
__host__ __device__ inline int swz16(int row) { return (row >> 1) & 3; }

template <int DT> __device__ inline f32x16_t mfma32(const uint4& a, const uint4& b, f32x16_t c) {
    if constexpr (DT == 1)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8_t, a), __builtin_bit_cast(h8_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf8_t, a), __builtin_bit_cast(bf8_t, b), c, 0, 0, 0);
}
// A: lane l holds row l % 16, k = 8 (l / 16) .. +7; B: column l % 16, the same k; D: column l % 16, rows 4 (l / 16) + e
template <int DT> __device__ inline f32x4_t mfma16(const uint4& a, const uint4& b, f32x4_t c) {
    if constexpr (DT == 1)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8_t, a), __builtin_bit_cast(h8_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8_t, a), __builtin_bit_cast(bf8_t, b), c, 0, 0, 0);
}

// The same MFMA with its accumulator in ordinary VGPRs.  The compiler keeps every accumulator of a kernel in one
// register class (here the 256 AGPRs); the tiles beyond those are accumulated through this form.  Its operands are
// tracked like any other instruction's (wait counts for the LDS reads that feed it); successive uses of one
// accumulator are a whole k-tile apart.
template <int DT> __device__ inline void mfma16_vgpr(const uint4& a, const uint4& b, f32x4_t& c) {
    const u32x4_t av = __builtin_bit_cast(u32x4_t, a), bv = __builtin_bit_cast(u32x4_t, b);
    if constexpr (DT == 1) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(c) : "v"(av), "v"(bv));
    else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(av), "v"(bv));
}

// 16-byte global -> LDS copy without a register stage: lane i's 16 bytes land at
// lds_addr + 16 i.  The LDS address goes through M0 and must be wave-uniform.
__device__ inline void gload_lds16(const void* g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory", "m0");
}
// The same with a wave-uniform 64-bit base and a 32-bit byte offset per lane.
__device__ inline void gload_lds16_base(const void* base, uint32_t lane_off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(lane_off), "s"(base)
                 : "memory", "m0");
}
typedef __attribute__((address_space(3))) u32x4_t lds_u32x4_t;
// 16-byte LDS read at an absolute LDS address (the dynamic LDS base is folded into the operand addresses once)
__device__ inline uint4 lds_read16(uint32_t addr) {
    const u32x4_t v = *(const lds_u32x4_t*)(uintptr_t)addr;
    return make_uint4(v.x, v.y, v.z, v.w);
}
template <int N> __device__ inline void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// byte offset of operand fragment f inside an LDS image: the W image holds the channels of a wave in order
// (fragment f = rows 16 f ..), the X image holds the token blocks of a wave interleaved with the other wave's
// (fragment f = the half f % 2 of the 32-token block f / 2, which sits 64 rows after the previous block)
__device__ constexpr int w_frag_off(int f) { return f * kFragBytes; }
__device__ constexpr int x_frag_off(int f) { return (64 * (f >> 1) + 16 * (f & 1)) * kRowBytes; }
// token row (within the tile) of the first token of X fragment f of the wave with token half th
__device__ inline int x_frag_row(int th, int f) { return th * 32 + 64 * (f >> 1) + 16 * (f & 1); }

template <int DT, int TF>
__global__ __launch_bounds__(kThreads) void apt_items_mfma_kernel(ItemParams p) {
    constexpr int HD = 128;
    constexpr int kTokFrags = TF, kTokTile = MfmaTile<TF>::kTokTile, kXChunks = MfmaTile<TF>::kXChunks;
    constexpr int kXTileBytes = MfmaTile<TF>::kXTileBytes, kStageLoads = MfmaTile<TF>::kStageLoads;
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mat = w >> 1, th = w & 1;
    const int d = p.d;
    const int nkt = d / kBK;                 // a multiple of 4: d is a multiple of 128
    const int64_t blk_bytes = (int64_t)p.bs * d * 2;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const uint32_t lds_w = lds_base + w * 1024;
    const int4* items = (const int4*)(p.plan + p.items_off);
    const int32_t* split_count = p.plan + APT_PW_HEADER;
    const int32_t* ws_offset = split_count + p.B;

    // ---- LDS layout: W stages 0..3 (16 KB each), X stages 0..3 (20 KB each), then the epilogue scratch
    float* scr = (float*)(lds + kStages * (kWTileBytes + kXTileBytes));
    float* p_lds = scr;                     // [kTokTile] softmax weights of the tile (per half, relative to its maximum)
    float* qs_lds = scr + kTokTile;         // [128] q * scale * log2(e)
    float* bk_lds = qs_lds + 128;           // [128]
    float* bv_lds = bk_lds + 128;           // [128]
    float* o_lds = bv_lds + 128;            // [2][128] per-half un-normalised output
    float* ml_lds = o_lds + 256;            // [2][2] per-half (m, l); [4], [5] = halves of q . b_K
    static_assert((kTokTile + 3 * 128 + 256 + 8) * 4 <= kMfmaScratch, "epilogue scratch too small");

    // This lane's 16 bytes of fragment 0, stage 0, in the W image (the channels of this wave) and in the X image
    // (the token blocks of this wave): row lane % 16 of the fragment, unit (lane / 16) ^ swz16(row); swz does not
    // change from fragment to fragment (their first rows are multiples of 16), so every other fragment and stage
    // is a constant offset away.
    // (computed per item, right before its k loop: kept across the epilogue they would sit in scratch)
    uint32_t w_base, x_base;
#define APT_OPERAND_ADDRESSES()                                                                             \
    {                                                                                                       \
        int ln_ = lane;                                                                                     \
        asm volatile("" : "+v"(ln_));                                                                       \
        const int l16_ = ln_ & 15, qd_ = ln_ >> 4;                                                          \
        const uint32_t off_ = l16_ * kRowBytes + ((qd_ ^ swz16(l16_)) * 16);                                  \
        w_base = lds_base + mat * 128 * kRowBytes + off_;                                                   \
        x_base = lds_base + kXImage + th * 32 * kRowBytes + off_;                                           \
    }

    // ---- this workgroup's share of the hidden-kind items
    const int G = gridDim.x, g = blockIdx.x;
    const int wpx = G >> 3;                                   // workgroups per queue (G is a multiple of 8)
    const int q_end = p.plan[APT_PW_QUEUE0 + (g & 7) + 1];
    int qi = p.plan[APT_PW_QUEUE0 + (g & 7)] + (g >> 3);

    // per-lane state of an item: kXChunks X row sources.  An X chunk of 1 KB is 16 rows; wave w
    // copies chunks w + 4 i: row 16 w + lane/4 + 64 i, LDS unit lane%4 = global unit (lane%4) ^ swz16(row)
    const int pu = lane & 3, r0 = 16 * w + (lane >> 2);
    int4 it = make_int4(0, 0, 0, 1);
    int32_t ids[kXChunks];
    auto lookup = [&](const int4& item, int32_t* out) {       // block ids of this lane's rows
#pragma unroll
        for (int i = 0; i < kXChunks; ++i) {
            int tok = item.z + r0 + 64 * i;
            tok = tok < item.w ? tok : item.w - 1;            // rows past the range repeat the last token (masked later)
            out[i] = p.block_tables[(int64_t)item.x * 2 * p.max_blocks + (tok >> p.log2_bs)];
        }
    };
    uint32_t xsrc[kXChunks];                                  // offsets from hidden_pages in 16-byte units
    const char* wsrc = nullptr;
#define APT_MAKE_SOURCES(XS, WS, ITEM, BLK)                                                                 \
    {                                                                                                       \
        _Pragma("unroll") for (int i_ = 0; i_ < kXChunks; ++i_) {                                           \
            const int row_ = r0 + 64 * i_;                                                                  \
            int tok_ = (ITEM).z + row_;                                                                     \
            tok_ = tok_ < (ITEM).w ? tok_ : (ITEM).w - 1;                                                   \
            XS[i_] = (uint32_t)(((int64_t)BLK[i_] * blk_bytes + ((int64_t)(tok_ & (p.bs - 1)) * d) * 2) >> 4) + \
                     (pu ^ swz16(row_));                                                                      \
        }                                                                                                   \
        WS = p.W_packed + (int64_t)(ITEM).y * nkt * kWTileBytes + w * 1024 + lane * 16;                     \
    }
    // copies chunk j (0..3: weights, 4..: X rows) of this wave's share of k-tile kt into stage st
    auto stage_chunk = [&](int kt, int st, int j) {
        if (j < 4)
            gload_lds16(wsrc + (int64_t)kt * kWTileBytes + j * 4096, lds_w + st * kWTileBytes + j * 4096);
        else
            gload_lds16(p.hidden_pages + (uint64_t)xsrc[j - 4] * 16 + kt * kRowBytes,
                        lds_w + kXImage + st * kXTileBytes + (j - 4) * 4096);
    };
#define APT_STAGE_FIRST(T0, T1)                                                                             \
    _Pragma("unroll") for (int t_ = (T0); t_ < (T1); ++t_) {                                                \
        _Pragma("unroll") for (int j_ = 0; j_ < kStageLoads; ++j_) stage_chunk(t_, t_, j_);                 \
    }

    bool have = qi < q_end;
    if (have) {
        it = items[qi];
        lookup(it, ids);
        APT_MAKE_SOURCES(xsrc, wsrc, it, ids)
        APT_STAGE_FIRST(0, 4)
    }

    // Accumulator tile (i, j): A-side fragment i (rows) x B-side fragment j (columns).  MAT 0 (K wave): A = W
    // fragments (NI = 8), B = X fragments (NJ = 2 per valid token block); MAT 1 (V wave): A = X, B = W.  The 64
    // tiles of the first 8 X fragments live in AGPRs (acc_a), the 16 tiles of X fragments 8 and 9 (the fifth
    // token block of the wave) in VGPRs (acc_v).
    constexpr int kAccV = kTokFrags > 8 ? 8 * (kTokFrags - 8) : 1;     // tiles accumulated in VGPRs (none for TF = 8)
    f32x4_t acc_a[64], acc_v[kAccV];
    // fr[set][..]: the NI A-side fragments, then the NJ B-side fragments of one k-tile.
    uint4 fr[2][8 + kTokFrags];
    // X fragment and W fragment of tile (I, J)
#define APT_XF(MAT, I, J) ((MAT) == 0 ? (J) : (I))
#define APT_WF(MAT, I, J) ((MAT) == 0 ? (I) : (J))
    // (indices are clamped so that the branch not taken never names an element outside its array)
#define APT_ACC_A_SAFE(MAT, I, J) acc_a[APT_XF(MAT, I, J) < 8 ? (I) * 8 + (J) : 0]
#define APT_ACC_V_SAFE(MAT, I, J) acc_v[APT_XF(MAT, I, J) < 8 ? 0 : (APT_XF(MAT, I, J) - 8) * 8 + APT_WF(MAT, I, J)]
#define APT_ACC_GET(MAT, I, J) (APT_XF(MAT, I, J) < 8 ? APT_ACC_A_SAFE(MAT, I, J) : APT_ACC_V_SAFE(MAT, I, J))
    // LDS address of operand slot R (0 .. NI + NJ - 1) in stage ST
#define APT_SLOT_ADDR(MAT, NI, R, ST)                                                                       \
    ((MAT) == 0 ? ((R) < (NI) ? w_base + w_frag_off(R) + (ST) * kWTileBytes                                 \
                              : x_base + x_frag_off((R) - (NI)) + (ST) * kXTileBytes)                       \
                : ((R) < (NI) ? x_base + x_frag_off(R) + (ST) * kXTileBytes                                 \
                              : w_base + w_frag_off((R) - (NI)) + (ST) * kWTileBytes))
    // MFMA index of a k-tile (after the operand reads of the next one) in front of which refill copy C is issued
#define APT_COPY_AT(C, NI, NJ) ((NI) + (NJ) + (C) * ((NI) * (NJ) - (NI) - (NJ)) / kStageLoads)
    // One k-tile, in stage ST, its operands already in register set ST % 2.  If another k-tile follows: all
    // waves meet (this wave's copies of the next k-tile have landed: at most WAITN younger copies may still be in
    // flight; every wave has all operands of THIS k-tile in registers, so its stage is no longer read), then the
    // next k-tile's operands are read into the other register set, one read per MFMA; after them, spread over the
    // remaining MFMAs, this stage is refilled with k-tile kt + 4.
#define APT_K_TILE(ST, STAGE, WAITN, NEXT, MAT, NI, NJ)                                                     \
    {                                                                                                       \
        if (NEXT) {                                                                                         \
            wait_vmcnt<WAITN>();                                                                            \
            __syncthreads();                                                                                \
        }                                                                                                   \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
        _Pragma("unroll") for (int m_ = 0; m_ < (NI) * (NJ); ++m_) {                                        \
            if (NEXT && m_ < (NI) + (NJ))                                                                   \
                fr[((ST) + 1) & 1][m_] = lds_read16(APT_SLOT_ADDR(MAT, NI, m_, ((ST) + 1) & 3));            \
            if (STAGE) {                                                                                    \
                _Pragma("unroll") for (int c_ = 0; c_ < kStageLoads; ++c_)                                  \
                    if (APT_COPY_AT(c_, NI, NJ) == m_) stage_chunk(kt + 4, ST, c_);                         \
            }                                                                                               \
            if (APT_XF(MAT, m_ / (NJ), m_ % (NJ)) < 8)                                                      \
                APT_ACC_A_SAFE(MAT, m_ / (NJ), m_ % (NJ)) =                                                 \
                    mfma16<DT>(fr[(ST) & 1][m_ / (NJ)], fr[(ST) & 1][(NI) + m_ % (NJ)],                     \
                               APT_ACC_A_SAFE(MAT, m_ / (NJ), m_ % (NJ)));                                  \
            else                                                                                            \
                mfma16_vgpr<DT>(fr[(ST) & 1][m_ / (NJ)], fr[(ST) & 1][(NI) + m_ % (NJ)],                    \
                                APT_ACC_V_SAFE(MAT, m_ / (NJ), m_ % (NJ)));                                 \
            __builtin_amdgcn_sched_barrier(0);                                                              \
        }                                                                                                   \
    }
    // The addresses used inside the k loop must be in registers with nothing pending behind them
    // when the loop starts: a reload the compiler still waits for inside the loop would also wait
    // for the staging copies.
#define APT_K_LOOP(MAT, NI, NJ)                                                                             \
    {                                                                                                       \
        asm volatile("" : "+v"(w_base), "+v"(x_base));                                                      \
        _Pragma("unroll") for (int i_ = 0; i_ < kXChunks; ++i_) asm volatile("" : "+v"(xsrc[i_]));          \
        asm volatile("" : "+v"(wsrc));                                                                      \
        _Pragma("unroll") for (int r_ = 0; r_ < (NI) + (NJ); ++r_) fr[0][r_] = lds_read16(APT_SLOT_ADDR(MAT, NI, r_, 0)); \
        int kt = 0;                                                                                         \
        for (; kt + 8 <= nkt; kt += 4) {                                                                    \
            APT_K_TILE(0, true, 2 * kStageLoads, true, MAT, NI, NJ)                                         \
            ++kt;                                                                                           \
            APT_K_TILE(1, true, 2 * kStageLoads, true, MAT, NI, NJ)                                         \
            ++kt;                                                                                           \
            APT_K_TILE(2, true, 2 * kStageLoads, true, MAT, NI, NJ)                                         \
            ++kt;                                                                                           \
            APT_K_TILE(3, true, 2 * kStageLoads, true, MAT, NI, NJ)                                         \
            kt -= 3;                                                                                        \
        }                                                                                                   \
        APT_K_TILE(0, false, 2 * kStageLoads, true, MAT, NI, NJ)   /* the last four k-tiles refill nothing */ \
        APT_K_TILE(1, false, kStageLoads, true, MAT, NI, NJ)                                                \
        APT_K_TILE(2, false, 0, true, MAT, NI, NJ)                                                          \
        APT_K_TILE(3, false, 0, false, MAT, NI, NJ)                                                         \
    }

    while (have) {
        const int r = it.x, h = it.y, t0 = it.z, nvalid = it.w - it.z;
        // block ids of the next item: on their way while this item's first copies land
        const int nqi = qi + wpx;
        const bool have_next = nqi < q_end;
        int4 itn = it;
        int32_t idsn[kXChunks];
#pragma unroll
        for (int i = 0; i < kXChunks; ++i) idsn[i] = 0;
        if (have_next) {
            itn = items[nqi];
            lookup(itn, idsn);
        }
        // per-item constants of the epilogue
        if (tid < HD) {
            const float qv = load_elem<DT>(p.q, ((int64_t)r * p.H + h) * HD + tid) * p.scale_log2e;
            const float bk = load_elem<DT>(p.b_K, (int64_t)h * HD + tid);
            qs_lds[tid] = qv;
            bk_lds[tid] = bk;
            bv_lds[tid] = load_elem<DT>(p.b_V, (int64_t)h * HD + tid);
            const float part = group_sum<64>(qv * bk);
            if (lane == 0) ml_lds[4 + w] = part;      // waves 0 and 1: halves of q . b_K
        }
        // valid token blocks of this wave: blocks 2 b + th below ceil(nvalid / 32)
        const int nvb = (nvalid + 31) >> 5;
        const int nb = (nvb - th + 1) >> 1;

#pragma unroll
        for (int i = 0; i < 64; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc_a[i][e] = 0.f;
        if constexpr (kTokFrags > 8) {
#pragma unroll
            for (int i = 0; i < kAccV; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc_v[i][e] = 0.f;
        }

        APT_OPERAND_ADDRESSES()
        // everything issued so far has to land here: the loads the compiler keeps track of (or the
        // wait counts it would place inside the k loop for them would also wait for the staging
        // copies) and with them the first four k-tiles
        wait_vmcnt<0>();
#pragma unroll
        for (int i = 0; i < kXChunks; ++i) asm volatile("" ::"v"(idsn[i]));
        asm volatile("" ::"v"(itn.x), "v"(itn.y), "v"(itn.z), "v"(itn.w));
        __syncthreads();
        // a short tile multiplies only the token blocks that hold valid tokens (at least one, so
        // that every wave runs the same barriers)
        bool full = false;
        if constexpr (kTokFrags == 10) {
            if (nb == 5) {
                full = true;
                if (mat == 0) APT_K_LOOP(0, 8, 10)
                else APT_K_LOOP(1, 10, 8)
            }
        }
        if (!full) {
            if (mat == 0) {
                if (nb == 4) APT_K_LOOP(0, 8, 8)
                else if (nb == 3) APT_K_LOOP(0, 8, 6)
                else if (nb == 2) APT_K_LOOP(0, 8, 4)
                else APT_K_LOOP(0, 8, 2)
            } else {
                if (nb == 4) APT_K_LOOP(1, 8, 8)
                else if (nb == 3) APT_K_LOOP(1, 6, 8)
                else if (nb == 2) APT_K_LOOP(1, 4, 8)
                else APT_K_LOOP(1, 2, 8)
            }
        }

        // stages 0..2 are free now (every wave has passed the last barrier of the k loop; stage 3
        // holds the last k-tile, which slower waves may still read): start the next item's first
        // three k-tiles, then finish this item
        if (have_next) {
            APT_MAKE_SOURCES(xsrc, wsrc, itn, idsn)
            APT_STAGE_FIRST(0, 3)
        }

        // ---- epilogue.  Register e of tile (i, j): row 4 (lane / 16) + e of the A-side fragment i,
        // column lane % 16 of the B-side fragment j.
        // lane-dependent LDS addresses of the epilogue are rebuilt here from values the compiler cannot see
        // through: hoisted out of the item loop they would stay live across the k loops and end up in scratch
        int ln = lane, td = tid;
        asm volatile("" : "+v"(ln), "+v"(td));
        const int l16 = ln & 15, qd = ln >> 4;
        if (mat == 0) {
            // K wave: rows = channels 16 i + 4 qd + e, columns = tokens of X fragment j
            const float qb = ml_lds[4] + ml_lds[5];
            float sp[kTokFrags];
#pragma unroll
            for (int j = 0; j < kTokFrags; ++j) sp[j] = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float4 q4 = *(const float4*)(qs_lds + 16 * i + 4 * qd);
#pragma unroll
                for (int j = 0; j < kTokFrags; ++j) {
                    const f32x4_t t = APT_ACC_GET(0, i, j);
                    sp[j] = fmaf(t[0], q4.x, sp[j]);
                    sp[j] = fmaf(t[1], q4.y, sp[j]);
                    sp[j] = fmaf(t[2], q4.z, sp[j]);
                    sp[j] = fmaf(t[3], q4.w, sp[j]);
                }
                // the accumulators are read out in small groups: read all at once they push every
                // long-lived value into scratch, and a scratch reload waits for the copies of the
                // next item's k-tiles that are in flight here
                __builtin_amdgcn_sched_barrier(0);
            }
            float m = kSentinel;
            bool ok[kTokFrags];
#pragma unroll
            for (int j = 0; j < kTokFrags; ++j) {
                sp[j] += __shfl_xor(sp[j], 16);
                sp[j] += __shfl_xor(sp[j], 32);
                ok[j] = x_frag_row(th, j) + l16 < nvalid;
                sp[j] = ok[j] ? sp[j] + qb : kSentinel;
                m = fmaxf(m, sp[j]);
            }
            m = group_max<16>(m);                     // the four lane groups hold the same scores
            float l = 0.f;
#pragma unroll
            for (int j = 0; j < kTokFrags; ++j) {
                const float pw = ok[j] ? fast_exp2(sp[j] - m) : 0.f;
                l += pw;
                if (qd == 0) p_lds[x_frag_row(th, j) + l16] = pw;
            }
            l = group_sum<16>(l);
            if (ln == 0) { ml_lds[th * 2] = m; ml_lds[th * 2 + 1] = l; }
        }
        __syncthreads();
        if (have_next) APT_STAGE_FIRST(3, 4)      // every wave has left the k loop: stage 3 is free too
        if (mat == 1) {
            // V wave: rows = tokens 4 qd + e of X fragment i, columns = channels 16 j + lane % 16
            float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < kTokFrags; ++i) {
                const float4 p4 = *(const float4*)(p_lds + x_frag_row(th, i) + 4 * qd);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const f32x4_t t = APT_ACC_GET(1, i, j);
                    o[j] = fmaf(t[0], p4.x, o[j]);
                    o[j] = fmaf(t[1], p4.y, o[j]);
                    o[j] = fmaf(t[2], p4.z, o[j]);
                    o[j] = fmaf(t[3], p4.w, o[j]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            const float l = ml_lds[th * 2 + 1];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                o[j] += __shfl_xor(o[j], 16);
                o[j] += __shfl_xor(o[j], 32);
                if (qd == 0) o_lds[th * 128 + 16 * j + l16] = fmaf(l, bv_lds[16 * j + l16], o[j]);
            }
        }
        __syncthreads();
        if (td < HD) {
            const float m0 = ml_lds[0], l0 = ml_lds[1], m1 = ml_lds[2], l1 = ml_lds[3];
            const float M = fmaxf(m0, m1);
            const float w0 = fast_exp2(m0 - M), w1 = fast_exp2(m1 - M);
            const int64_t slot = ((int64_t)ws_offset[r] + t0 / p.hidden_chunk) * p.H + h;
            p.ws_acc[slot * HD + td] = o_lds[td] * w0 + o_lds[128 + td] * w1;
            if (td == 0) p.ws_ml[slot] = make_float2(M, l0 * w0 + l1 * w1);
        }
        have = have_next;
        qi = nqi;
        it = itn;
    }
#undef APT_K_LOOP
#undef APT_K_TILE
#undef APT_COPY_AT
#undef APT_SLOT_ADDR
#undef APT_ACC_GET
#undef APT_ACC_V_SAFE
#undef APT_ACC_A_SAFE
#undef APT_WF
#undef APT_XF
#undef APT_STAGE_FIRST
#undef APT_OPERAND_ADDRESSES
#undef APT_MAKE_SOURCES

    // ---- then a share of the KV-kind items, longest first
    __syncthreads();
    // handed out one by one, so that workgroups that finish their hidden-kind share early take more
    int* ticket_lds = (int*)(lds + kStages * (kWTileBytes + kXTileBytes));
    for (;;) {
        if (tid == 0) *ticket_lds = atomicAdd(p.kv_ticket, 1);
        __syncthreads();
        const int i = p.n_hidden_items + *ticket_lds;
        if (i >= p.n_items) break;
        const int4 kv = items[i];
        kv_item<DT, HD>(p, kv.x, kv.y, kv.z, kv.w, lds);
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------
// the items kernel, one workgroup per item.  HIMPL: 0 = no hidden-kind items in the plan,
// 1 = plain-ALU hidden kernel.  (Plans with MFMA hidden items run apt_items_mfma_kernel.)
// ---------------------------------------------------------------------------------
template <int DT, int HD, int HIMPL>
__global__ __launch_bounds__(kThreads) void apt_items_kernel(ItemParams p) {
    extern __shared__ __align__(16) char lds[];
    const int item = blockIdx.x + p.item_base;
    if (item >= p.n_items) return;
    const int4 it = ((const int4*)(p.plan + p.items_off))[item];
    if (item < p.n_hidden_items) {
        if constexpr (HIMPL == 1) hidden_item_valu<DT, HD>(p, it.x, it.y, it.z, it.w, lds);
    } else {
        kv_item<DT, HD>(p, it.x, it.y, it.z, it.w, lds);
    }
}

// ---------------------------------------------------------------------------------
// merge kernel: out[r][h][c] = sum_s acc_s[c] 2^(m_s - M) / sum_s l_s 2^(m_s - M)
// ---------------------------------------------------------------------------------
template <int ODT>
__global__ __launch_bounds__(kThreads) void apt_merge_kernel(const int32_t* plan, const float* ws_acc, const float2* ws_ml,
                                                             char* out, int B, int H, int HD, int32_t* kv_ticket,
                                                             int skip_hidden) {
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (gid == 0) *kv_ticket = 0;           // the item kernel of this call is done: ready for the next call
    if (gid >= (int64_t)B * H * HD) return;
    const int c = (int)(gid % HD);
    const int64_t pair = gid / HD;
    const int h = (int)(pair % H), r = (int)(pair / H);
    const int32_t* split_count = plan + APT_PW_HEADER + APT_PA_SPLIT_COUNT * B;
    const int32_t* ws_offset = plan + APT_PW_HEADER + APT_PA_WS_OFFSET * B;
    // absorbed-weight path: the outputs of hidden-kind requests are already written
    if (skip_hidden && plan[APT_PW_HEADER + APT_PA_KIND * B + r] == APT_KIND_HIDDEN) return;
    const int ns = split_count[r];
    const int64_t base = (int64_t)ws_offset[r] * H + h;
    float M = kSentinel;
    for (int s = 0; s < ns; ++s) M = fmaxf(M, ws_ml[base + (int64_t)s * H].x);
    float L = 0.f, A = 0.f;
    for (int s = 0; s < ns; ++s) {
        const int64_t slot = base + (int64_t)s * H;
        const float2 ml = ws_ml[slot];
        const float wgt = fast_exp2(ml.x - M);
        L = fmaf(ml.y, wgt, L);
        A = fmaf(ws_acc[slot * HD + c], wgt, A);
    }
    const float o = A / L;
    if constexpr (ODT == 0) ((float*)out)[gid] = o;
    else if constexpr (ODT == 1) ((_Float16*)out)[gid] = (_Float16)o;
    else ((uint16_t*)out)[gid] = f32_to_bf16_rne(o);
}

// ---------------------------------------------------------------------------------
// weight packing for the MFMA kernel (one-off per layer)
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void apt_pack_kernel(const uint16_t* W_K, const uint16_t* W_V, uint4* packed,
                                                            int d, int H) {
    // one thread per 16-byte unit; consecutive threads take consecutive channels so
    // that the strided reads of W coalesce
    const int nkt = d / kBK;
    constexpr int units = kBK / 8;                      // 16-byte units per row
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t total = (int64_t)H * nkt * 256 * units;
    if (gid >= total) return;
    const int row = (int)(gid % 256);
    const int c = (int)((gid / 256) % units);
    const int kt = (int)((gid / (256 * units)) % nkt);
    const int h = (int)(gid / (256 * units * (int64_t)nkt));
    const uint16_t* W = row < 128 ? W_K : W_V;
    const int ch = h * 128 + (row & 127);
    const int k0 = kt * kBK + c * 8;
    uint16_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = W[(int64_t)(k0 + e) * d + ch];
    uint4 o;
    o.x = v[0] | ((uint32_t)v[1] << 16);
    o.y = v[2] | ((uint32_t)v[3] << 16);
    o.z = v[4] | ((uint32_t)v[5] << 16);
    o.w = v[6] | ((uint32_t)v[7] << 16);
    packed[((int64_t)h * nkt + kt) * (256 * units) + row * units + (c ^ swz16(row))] = o;
}

// Cache append: one workgroup per request, 16-byte units.  A unit never straddles a head
// (head_dim * element size is a multiple of 16).
__global__ __launch_bounds__(kThreads) void apt_append_kernel(const char* x_new, const char* k_new, const char* v_new,
                                                              char* k_pages, char* v_pages, char* hidden_pages,
                                                              const int32_t* block_tables, const int32_t* ctx_lens,
                                                              const uint8_t* cache_kind, int d, int hd, int bs, int log2_bs,
                                                              int max_blocks, int eb) {
    const int r = blockIdx.x;
    const int j = ctx_lens[r] - 1;
    if (j < 0) return;
    const int slot = j & (bs - 1);
    const int64_t blk_bytes = (int64_t)bs * d * eb;
    const int row_units = d * eb / 16;
    const int64_t e0 = (int64_t)r * 2 * max_blocks + (j >> log2_bs);
    if (cache_kind[r] == APT_KIND_HIDDEN) {
        char* dst = hidden_pages + (int64_t)block_tables[e0] * blk_bytes + (int64_t)slot * d * eb;
        for (int u = threadIdx.x; u < row_units; u += kThreads)
            *(uint4*)(dst + (int64_t)u * 16) = *(const uint4*)(x_new + ((int64_t)r * row_units + u) * 16);
    } else {
        char* kd = k_pages + (int64_t)block_tables[e0] * blk_bytes;
        char* vd = v_pages + (int64_t)block_tables[e0 + max_blocks] * blk_bytes;
        const int head_units = hd * eb / 16;
        for (int u = threadIdx.x; u < row_units; u += kThreads) {
            const int h = u / head_units, cu = u % head_units;
            const int64_t off = (((int64_t)h * bs + slot) * hd) * eb + (int64_t)cu * 16;
            *(uint4*)(kd + off) = *(const uint4*)(k_new + ((int64_t)r * row_units + u) * 16);
            *(uint4*)(vd + off) = *(const uint4*)(v_new + ((int64_t)r * row_units + u) * 16);
        }
    }
}

// Cache write of a run of new tokens per request (prefill, or several decoded tokens at once): grid
// (request, group of kWriteTokens new tokens), 16-byte units as in the append kernel.
constexpr int kWriteTokens = 8;
__global__ __launch_bounds__(kThreads) void apt_write_kernel(const int32_t* new_offsets, const char* x_new, const char* k_new,
                                                             const char* v_new, char* k_pages, char* v_pages,
                                                             char* hidden_pages, const int32_t* block_tables,
                                                             const int32_t* ctx_lens, const uint8_t* cache_kind, int d, int hd,
                                                             int bs, int log2_bs, int max_blocks, int eb) {
    const int r = blockIdx.x;
    const int row0 = new_offsets[r], n_new = new_offsets[r + 1] - row0;
    const int first = ctx_lens[r] - n_new;              // position of the first new token
    if (n_new <= 0 || first < 0) return;                // more new tokens than the request holds: nothing is written
    const int64_t blk_bytes = (int64_t)bs * d * eb;
    const int row_units = d * eb / 16, head_units = hd * eb / 16;
    const bool hidden = cache_kind[r] == APT_KIND_HIDDEN;
    for (int t = blockIdx.y * kWriteTokens; t < min(n_new, (int)(blockIdx.y + 1) * kWriteTokens); ++t) {
        const int j = first + t, slot = j & (bs - 1);
        const int64_t e0 = (int64_t)r * 2 * max_blocks + (j >> log2_bs);
        const int64_t src = (int64_t)(row0 + t) * row_units;
        if (hidden) {
            char* dst = hidden_pages + (int64_t)block_tables[e0] * blk_bytes + (int64_t)slot * d * eb;
            for (int u = threadIdx.x; u < row_units; u += kThreads)
                *(uint4*)(dst + (int64_t)u * 16) = *(const uint4*)(x_new + (src + u) * 16);
        } else {
            char* kd = k_pages + (int64_t)block_tables[e0] * blk_bytes;
            char* vd = v_pages + (int64_t)block_tables[e0 + max_blocks] * blk_bytes;
            for (int u = threadIdx.x; u < row_units; u += kThreads) {
                const int h = u / head_units, cu = u % head_units;
                const int64_t off = (((int64_t)h * bs + slot) * hd) * eb + (int64_t)cu * 16;
                *(uint4*)(kd + off) = *(const uint4*)(k_new + (src + u) * 16);
                *(uint4*)(vd + off) = *(const uint4*)(v_new + (src + u) * 16);
            }
        }
    }
}

__global__ __launch_bounds__(kThreads) void apt_copy_kernel(uint4* dst, const uint4* src, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (; i < n; i += stride) dst[i] = src[i];
}

// Register-only MFMA loop: 4 waves per workgroup, a 128 x 128 accumulator tile per wave (256 registers), no
// memory traffic.  Measures the rate the matrix pipes sustain.  With random_operands the operand registers
// hold values of magnitude ~1 with random mantissas and signs (what real activations look like to the
// multipliers) instead of constants.  VARIANT 0 / 2: 16 independent 32x32x16 MFMAs per iteration (fp16 /
// bf16); 1 / 3: 64 independent 16x16x32 MFMAs per iteration (fp16 / bf16; twice the flops per iteration).
template <int VARIANT>
__global__ __launch_bounds__(kThreads) void apt_mfma_probe_kernel(float* out, int iters, int random_operands) {
    constexpr bool kSmall = (VARIANT & 1) != 0;          // 16x16x32 tiles
    constexpr int DT = (VARIANT & 2) ? 2 : 1;
    constexpr int NF = kSmall ? 8 : 4;                   // operand fragments per side
    uint4 a[NF], b[NF];
    uint32_t x = (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u + 12345u);
    const uint32_t one = DT == 1 ? 0x3c003c00u : 0x3f803f80u, half = DT == 1 ? 0x38003800u : 0x3f003f00u;
    const uint32_t keep = DT == 1 ? 0x83ff83ffu : 0x807f807fu;      // sign and mantissa bits
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        a[i] = make_uint4(one, one, one, one);
        b[i] = make_uint4(half, half, half, half);
        if (random_operands) {
            auto nxt = [&]() { x ^= x << 13; x ^= x >> 17; x ^= x << 5; return (x & keep) | one; };
            a[i] = make_uint4(nxt(), nxt(), nxt(), nxt());
            b[i] = make_uint4(nxt(), nxt(), nxt(), nxt());
        }
    }
    float sum = 0.f;
    if constexpr (!kSmall) {
        f32x16_t acc[16];
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i * 4 + j] = mfma32<DT>(a[i], b[j], acc[i * 4 + j]);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) sum += acc[i][e];
    } else {
        f32x4_t acc[64];
#pragma unroll
        for (int i = 0; i < 64; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][e] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if constexpr (DT == 1)
                        acc[i * 8 + j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8_t, a[i]),
                                                                                __builtin_bit_cast(h8_t, b[j]), acc[i * 8 + j], 0, 0, 0);
                    else
                        acc[i * 8 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8_t, a[i]),
                                                                                 __builtin_bit_cast(bf8_t, b[j]), acc[i * 8 + j], 0, 0, 0);
                }
        }
#pragma unroll
        for (int i = 0; i < 64; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) sum += acc[i][e];
    }
    out[(int64_t)blockIdx.x * kThreads + threadIdx.x] = sum;
}

// ---------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------
template <int DT, int HD, int HIMPL>
int launch_items(const ItemParams& p, size_t lds_bytes, hipStream_t st) {
    auto kern = apt_items_kernel<DT, HD, HIMPL>;
    hipLaunchKernelGGL(kern, dim3(p.n_items - p.item_base), dim3(kThreads), lds_bytes, st, p);
    return hipGetLastError() == hipSuccess ? APT_OK : APT_EHIP;
}

#include "apt_absorbed.inc"

// persistent launch: one workgroup per compute unit, a multiple of 8
template <int DT>
int launch_mfma(const ItemParams& p, int n_wg, hipStream_t st) {
    if (p.hidden_chunk == MfmaTile<10>::kTokTile)
        hipLaunchKernelGGL((apt_items_mfma_kernel<DT, 10>), dim3(n_wg), dim3(kThreads), MfmaTile<10>::kLds, st, p);
    else if (p.hidden_chunk == MfmaTile<8>::kTokTile)
        hipLaunchKernelGGL((apt_items_mfma_kernel<DT, 8>), dim3(n_wg), dim3(kThreads), MfmaTile<8>::kLds, st, p);
    else
        return APT_ESHAPE;
    return hipGetLastError() == hipSuccess ? APT_OK : APT_EHIP;
}

template <int DT, int HD>
int launch_items_impl(const ItemParams& p_in, int himpl, char* out, int out_dtype, int n_wg, hipStream_t st) {
    constexpr int EB = Elt<DT>::bytes;
    constexpr int LPR = HD * EB / 16;
    constexpr int G = 4 * (64 / LPR);
    const size_t kv_lds = (size_t)(2 * G + G * HD) * 4;
    ItemParams p = p_in;
    if (p.n_hidden_items == 0) return launch_items<DT, HD, 0>(p, kv_lds, st);
    if (himpl == APT_HIDDEN_ABSORBED) {
        const int rc = launch_absorbed<DT>(p, out, out_dtype, HD, st);
        if (rc || p.n_hidden_items == p.n_items) return rc;
        p.item_base = p.n_hidden_items;          // the KV-kind items, one workgroup each
        return launch_items<DT, HD, 0>(p, kv_lds, st);
    }
    if (himpl == APT_HIDDEN_VALU) {
        size_t v = (size_t)(2 * p.hidden_chunk * (HD + 1) + 64 + 2) * 4;
        return launch_items<DT, HD, 1>(p, v > kv_lds ? v : kv_lds, st);
    }
    if constexpr (DT != 0 && HD == 128) {
        return launch_mfma<DT>(p, n_wg, st);
    }
    return APT_ESHAPE;
}

// ---------------------------------------------------------------------------------
// per-device set-up: made once per device under a mutex, read-only afterwards
// ---------------------------------------------------------------------------------
struct DeviceState {
    bool ready = false;
    int n_wg = 0;             // workgroups of the persistent MFMA launch
    void* scratch_ptr = nullptr;  // this device's copy of the static workspace
};
constexpr int kMaxDevices = 64;
std::mutex g_setup_mutex;
DeviceState g_devices[kMaxDevices];

template <typename K> bool raise_lds_limit(K kern) {
    return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) == hipSuccess;
}

int device_setup(const DeviceState** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return APT_EHIP;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    DeviceState& ds = g_devices[dev];
    if (!ds.ready) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return APT_EHIP;
        ds.n_wg = cus >= 8 ? (cus / 8) * 8 : 8;
        // every kernel that can be launched with more than 64 KB of dynamic LDS
        const bool ok = raise_lds_limit(apt_items_mfma_kernel<1, 8>) && raise_lds_limit(apt_items_mfma_kernel<2, 8>) &&
                        raise_lds_limit(apt_items_mfma_kernel<1, 10>) && raise_lds_limit(apt_items_mfma_kernel<2, 10>) &&
                        raise_lds_limit(apt_items_kernel<0, 64, 1>) && raise_lds_limit(apt_items_kernel<0, 128, 1>) &&
                        raise_lds_limit(apt_items_kernel<1, 64, 1>) && raise_lds_limit(apt_items_kernel<1, 128, 1>) &&
                        raise_lds_limit(apt_items_kernel<2, 64, 1>) && raise_lds_limit(apt_items_kernel<2, 128, 1>) &&
                        raise_lds_limit(apt_absorb_score_kernel<0>) && raise_lds_limit(apt_absorb_pv_kernel<0>) &&
                        raise_lds_limit(apt_absorb_score_mfma_kernel<1>) && raise_lds_limit(apt_absorb_score_mfma_kernel<2>) &&
                        raise_lds_limit(apt_absorb_pv_mfma_kernel<1>) && raise_lds_limit(apt_absorb_pv_mfma_kernel<2>);
        if (!ok) return APT_EHIP;
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return APT_EHIP;
        ds.scratch_ptr = ptr;
        ds.ready = true;
    }
    if (out) *out = &ds;
    return APT_OK;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

extern "C" int apt_init(void) { return device_setup(nullptr); }

extern "C" int apt_plan_upload(const void* plan_host, void* plan_dev, void* stream) {
    apt_plan_info info;
    int rc = apt_plan_get_info(plan_host, &info);
    if (rc) return rc;
    if (!plan_dev) return APT_EINVAL;
    if (hipMemcpyAsync(plan_dev, plan_host, info.plan_bytes, hipMemcpyHostToDevice, (hipStream_t)stream) != hipSuccess)
        return APT_EHIP;
    return APT_OK;
}

extern "C" int apt_packed_weight_bytes(const apt_shape* s, size_t* bytes) {
    apt_resolved rs;
    int rc = apt_resolve(s, &rs);
    if (rc) return rc;
    if (!bytes) return APT_EINVAL;
    *bytes = (size_t)2 * rs.s.d_model * rs.s.d_model * rs.elem_bytes;
    return APT_OK;
}

extern "C" int apt_pack_weights(const apt_shape* s, const void* W_K, const void* W_V, void* packed, void* stream) {
    apt_resolved rs;
    int rc = apt_resolve(s, &rs);
    if (rc) return rc;
    if (!W_K || !W_V || !packed) return APT_EINVAL;
    if (rs.s.hidden_impl != APT_HIDDEN_MFMA) return APT_ESHAPE;
    const int d = rs.s.d_model, H = rs.s.n_heads;
    const int64_t total = (int64_t)H * (d / kBK) * 256 * (kBK / 8);
    const int64_t blocks = (total + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(apt_pack_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream,
                       (const uint16_t*)W_K, (const uint16_t*)W_V, (uint4*)packed, d, H);
    return hipGetLastError() == hipSuccess ? APT_OK : APT_EHIP;
}

extern "C" int apt_cache_append(const apt_shape* s, int B, const void* x_new, const void* k_new, const void* v_new,
                                void* k_pages, void* v_pages, void* hidden_pages, const int32_t* block_tables,
                                const int32_t* ctx_lens_dev, const uint8_t* cache_kind_dev, void* stream) {
    apt_resolved rs;
    int rc = apt_resolve(s, &rs);
    if (rc) return rc;
    if (B < 1 || !block_tables || !ctx_lens_dev || !cache_kind_dev) return APT_EINVAL;
    if (!x_new && !k_new && !v_new) return APT_EINVAL;
    if ((x_new && !hidden_pages) || ((k_new || v_new) && (!k_new || !v_new || !k_pages || !v_pages))) return APT_EINVAL;
    if (!aligned16(x_new) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_pages) || !aligned16(v_pages) ||
        !aligned16(hidden_pages))
        return APT_EINVAL;
    int log2_bs = 0;
    while ((1 << log2_bs) < rs.s.block_size) ++log2_bs;
    hipLaunchKernelGGL(apt_append_kernel, dim3(B), dim3(kThreads), 0, (hipStream_t)stream, (const char*)x_new,
                       (const char*)k_new, (const char*)v_new, (char*)k_pages, (char*)v_pages, (char*)hidden_pages,
                       block_tables, ctx_lens_dev, cache_kind_dev, rs.s.d_model, rs.s.head_dim, rs.s.block_size, log2_bs,
                       rs.s.max_blocks_per_req, rs.elem_bytes);
    return hipGetLastError() == hipSuccess ? APT_OK : APT_EHIP;
}

extern "C" int apt_cache_write(const apt_shape* s, int B, const int32_t* new_offsets_dev, int32_t max_new_tokens,
                               const void* x_new, const void* k_new, const void* v_new, void* k_pages, void* v_pages,
                               void* hidden_pages, const int32_t* block_tables, const int32_t* ctx_lens_dev,
                               const uint8_t* cache_kind_dev, void* stream) {
    apt_resolved rs;
    int rc = apt_resolve(s, &rs);
    if (rc) return rc;
    if (B < 1 || max_new_tokens < 1 || !new_offsets_dev || !block_tables || !ctx_lens_dev || !cache_kind_dev) return APT_EINVAL;
    if (!x_new && !k_new && !v_new) return APT_EINVAL;
    if ((x_new && !hidden_pages) || ((k_new || v_new) && (!k_new || !v_new || !k_pages || !v_pages))) return APT_EINVAL;
    if (!aligned16(x_new) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_pages) || !aligned16(v_pages) ||
        !aligned16(hidden_pages))
        return APT_EINVAL;
    int log2_bs = 0;
    while ((1 << log2_bs) < rs.s.block_size) ++log2_bs;
    const unsigned groups = (unsigned)((max_new_tokens + kWriteTokens - 1) / kWriteTokens);
    if (groups > 65535u) return APT_ERANGE;
    hipLaunchKernelGGL(apt_write_kernel, dim3(B, groups), dim3(kThreads), 0, (hipStream_t)stream, new_offsets_dev,
                       (const char*)x_new, (const char*)k_new, (const char*)v_new, (char*)k_pages, (char*)v_pages,
                       (char*)hidden_pages, block_tables, ctx_lens_dev, cache_kind_dev, rs.s.d_model, rs.s.head_dim,
                       rs.s.block_size, log2_bs, rs.s.max_blocks_per_req, rs.elem_bytes);
    return hipGetLastError() == hipSuccess ? APT_OK : APT_EHIP;
}

extern "C" int apt_copy_bytes(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || bytes == 0 || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return APT_EINVAL;
    const int64_t n = (int64_t)(bytes / 16);
    int64_t blocks = (n + kThreads - 1) / kThreads;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(apt_copy_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream,
                       (uint4*)dst, (const uint4*)src, n);
    return hipGetLastError() == hipSuccess ? APT_OK : APT_EHIP;
}

extern "C" int apt_probe_mfma(void* out, int n_workgroups, int iters, int random_operands, int variant, void* stream) {
    if (!out || n_workgroups < 1 || iters < 1 || variant < 0 || variant > 3) return APT_EINVAL;
    const dim3 grid(n_workgroups), block(kThreads);
    hipStream_t st = (hipStream_t)stream;
    if (variant == 0) hipLaunchKernelGGL(apt_mfma_probe_kernel<0>, grid, block, 0, st, (float*)out, iters, random_operands);
    else if (variant == 1) hipLaunchKernelGGL(apt_mfma_probe_kernel<1>, grid, block, 0, st, (float*)out, iters, random_operands);
    else if (variant == 2) hipLaunchKernelGGL(apt_mfma_probe_kernel<2>, grid, block, 0, st, (float*)out, iters, random_operands);
    else hipLaunchKernelGGL(apt_mfma_probe_kernel<3>, grid, block, 0, st, (float*)out, iters, random_operands);
    return hipGetLastError() == hipSuccess ? APT_OK : APT_EHIP;
}

// The attention step behind all three entry points.  static_ws: the partials go to this device's static workspace
// (workspace / workspace_bytes are ignored) and nothing may be allocated.
static int decode_attn(const apt_shape* s, const void* plan_host, void* plan_dev,
                       const void* q, const void* k_pages, const void* v_pages, const void* hidden_pages,
                       const void* W_K, const void* W_V, const void* W_packed,
                       const void* b_K, const void* b_V, const int32_t* block_tables,
                       void* out, void* workspace, size_t workspace_bytes, bool static_ws, void* stream,
                       void* ev_begin, void* ev_end) {
    apt_resolved rs;
    int rc = apt_resolve(s, &rs);
    if (rc) return rc;
    if (!plan_host || !plan_dev || !q || !block_tables || !out || (!workspace && !static_ws)) return APT_EINVAL;
    if (static_ws && rs.s.hidden_impl == APT_HIDDEN_ABSORBED) return APT_ESHAPE;
    if (static_ws) workspace_bytes = APT_STATIC_WORKSPACE_BYTES;
    const int32_t* pw = (const int32_t*)plan_host;
    if (pw[APT_PW_MAGIC] != APT_PLAN_MAGIC) return APT_EINVAL;
    // the plan must have been made for this shape
    if (pw[APT_PW_HEADS] != rs.s.n_heads || pw[APT_PW_HEAD_DIM] != rs.s.head_dim || pw[APT_PW_HCHUNK] != rs.s.hidden_chunk ||
        pw[APT_PW_HIMPL] != rs.s.hidden_impl || pw[APT_PW_D_MODEL] != rs.s.d_model ||
        pw[APT_PW_BLOCK_SIZE] != rs.s.block_size || pw[APT_PW_MAX_BLOCKS] != rs.s.max_blocks_per_req ||
        pw[APT_PW_DTYPE] != rs.s.dtype)
        return APT_ESHAPE;
    // KV-kind range length: the caller's, or the planner's choice for this batch when the caller left it open
    const int kv_chunk = pw[APT_PW_KCHUNK];
    if (rs.kv_auto ? (kv_chunk < rs.s.kv_chunk || kv_chunk > APT_MAX_AUTO_KV_CHUNK || !apt_kv_chunk_ok(kv_chunk, rs.s.block_size))
                   : kv_chunk != rs.s.kv_chunk)
        return APT_ESHAPE;
    const int n_items = pw[APT_PW_NITEMS], n_hidden = pw[APT_PW_NHIDDEN];
    const int B = pw[APT_PW_BATCH];
    const int64_t hidden_tokens = ((int64_t)pw[APT_PW_HTOK_HI] << 32) | (uint32_t)pw[APT_PW_HTOK_LO];
    const apt_ws_layout L = apt_ws_sections(pw[APT_PW_NPARTIALS], rs.s.n_heads, rs.s.head_dim, rs.s.hidden_impl,
                                            pw[APT_PW_NHIDREQ], hidden_tokens, n_hidden, rs.s.d_model, rs.s.dtype);
    if (workspace_bytes < L.total) return APT_EWORKSPACE;
    // 16-byte vector loads and stores: every base pointer has to be 16-byte aligned
    if ((!static_ws && !aligned16(workspace)) || !aligned16(q) || !aligned16(k_pages) || !aligned16(v_pages) || !aligned16(hidden_pages) ||
        !aligned16(W_K) || !aligned16(W_V) || !aligned16(W_packed) || !aligned16(b_K) || !aligned16(b_V) || !aligned16(plan_dev))
        return APT_EINVAL;
    if (n_hidden < n_items && (!k_pages || !v_pages)) return APT_EINVAL;
    if (n_hidden > 0) {
        if (!hidden_pages || !b_K || !b_V) return APT_EINVAL;
        if (rs.s.hidden_impl == APT_HIDDEN_MFMA && !W_packed) return APT_EINVAL;
        if (rs.s.hidden_impl != APT_HIDDEN_MFMA && (!W_K || !W_V)) return APT_EINVAL;
    }
    int log2_bs = 0;
    while ((1 << log2_bs) < rs.s.block_size) ++log2_bs;
    // every argument is checked: now the device (first call on a device: its one-off set-up)
    const DeviceState* ds = nullptr;
    rc = device_setup(&ds);
    if (rc) return rc;
    if (static_ws) workspace = ds->scratch_ptr;

    ItemParams p;
    p.plan = (const int32_t*)plan_dev;
    p.kv_ticket = (int32_t*)plan_dev + APT_PW_KV_TICKET;
    p.q = (const char*)q;
    p.k_pages = (const char*)k_pages;
    p.v_pages = (const char*)v_pages;
    p.hidden_pages = (const char*)hidden_pages;
    p.W_K = (const char*)W_K;
    p.W_V = (const char*)W_V;
    p.W_packed = (const char*)W_packed;
    p.b_K = (const char*)b_K;
    p.b_V = (const char*)b_V;
    p.block_tables = block_tables;
    char* const ws = (char*)workspace;
    p.ws_acc = (float*)(ws + L.acc);
    p.ws_ml = (float2*)(ws + L.ml);
    p.ab_qt = (float*)(ws + L.qt);
    p.ab_cb = (float*)(ws + L.cb);
    p.ab_s = (float*)(ws + L.s);
    p.ab_ml = (float2*)(ws + L.stat);
    p.ab_yp = (float*)(ws + L.yp);
    p.ab_op = (float*)(ws + L.op);
    p.ab_pp = ws + L.pp;
    p.ab_tokens = hidden_tokens;
    p.n_hid_req = pw[APT_PW_NHIDREQ];
    p.item_base = 0;
    p.B = B; p.H = rs.s.n_heads; p.d = rs.s.d_model; p.bs = rs.s.block_size; p.log2_bs = log2_bs;
    p.max_blocks = rs.s.max_blocks_per_req;
    p.n_items = n_items; p.n_hidden_items = n_hidden;
    p.hidden_chunk = rs.s.hidden_chunk; p.kv_chunk = kv_chunk; p.items_off = pw[APT_PW_ITEMS_OFF];
    p.scale_log2e = rs.s.softmax_scale * 1.4426950408889634f;
    hipStream_t st = (hipStream_t)stream;

    const int dt = rs.s.dtype, hd = rs.s.head_dim, hi = rs.s.hidden_impl;
    if (ev_begin && hipEventRecord((hipEvent_t)ev_begin, st) != hipSuccess) return APT_EHIP;
    if (dt == APT_F32 && hd == 64) rc = launch_items_impl<0, 64>(p, hi, (char*)out, rs.s.out_dtype, ds->n_wg, st);
    else if (dt == APT_F32 && hd == 128) rc = launch_items_impl<0, 128>(p, hi, (char*)out, rs.s.out_dtype, ds->n_wg, st);
    else if (dt == APT_F16 && hd == 64) rc = launch_items_impl<1, 64>(p, hi, (char*)out, rs.s.out_dtype, ds->n_wg, st);
    else if (dt == APT_F16 && hd == 128) rc = launch_items_impl<1, 128>(p, hi, (char*)out, rs.s.out_dtype, ds->n_wg, st);
    else if (dt == APT_BF16 && hd == 64) rc = launch_items_impl<2, 64>(p, hi, (char*)out, rs.s.out_dtype, ds->n_wg, st);
    else rc = launch_items_impl<2, 128>(p, hi, (char*)out, rs.s.out_dtype, ds->n_wg, st);
    if (rc) return rc;
    if (ev_end && hipEventRecord((hipEvent_t)ev_end, st) != hipSuccess) return APT_EHIP;

    const int skip_hidden = hi == APT_HIDDEN_ABSORBED;
    const int64_t total = (int64_t)B * rs.s.n_heads * hd;
    const unsigned blocks = (unsigned)((total + kThreads - 1) / kThreads);
    if (rs.s.out_dtype == APT_F32)
        hipLaunchKernelGGL(apt_merge_kernel<0>, dim3(blocks), dim3(kThreads), 0, st, p.plan, p.ws_acc, p.ws_ml, (char*)out, B, rs.s.n_heads, hd, p.kv_ticket, skip_hidden);
    else if (rs.s.out_dtype == APT_F16)
        hipLaunchKernelGGL(apt_merge_kernel<1>, dim3(blocks), dim3(kThreads), 0, st, p.plan, p.ws_acc, p.ws_ml, (char*)out, B, rs.s.n_heads, hd, p.kv_ticket, skip_hidden);
    else
        hipLaunchKernelGGL(apt_merge_kernel<2>, dim3(blocks), dim3(kThreads), 0, st, p.plan, p.ws_acc, p.ws_ml, (char*)out, B, rs.s.n_heads, hd, p.kv_ticket, skip_hidden);
    return hipGetLastError() == hipSuccess ? APT_OK : APT_EHIP;
}

extern "C" int apt_hybrid_decode_attn_timed(const apt_shape* s, const void* plan_host, void* plan_dev,
                                            const void* q, const void* k_pages, const void* v_pages, const void* hidden_pages,
                                            const void* W_K, const void* W_V, const void* W_packed,
                                            const void* b_K, const void* b_V, const int32_t* block_tables,
                                            void* out, void* workspace, size_t workspace_bytes, void* stream,
                                            void* ev_begin, void* ev_end) {
    return decode_attn(s, plan_host, plan_dev, q, k_pages, v_pages, hidden_pages, W_K, W_V, W_packed, b_K, b_V,
                       block_tables, out, workspace, workspace_bytes, false, stream, ev_begin, ev_end);
}

extern "C" int apt_hybrid_decode_attn(const apt_shape* s, const void* plan_host, void* plan_dev,
                                      const void* q, const void* k_pages, const void* v_pages, const void* hidden_pages,
                                      const void* W_K, const void* W_V, const void* W_packed,
                                      const void* b_K, const void* b_V, const int32_t* block_tables,
                                      void* out, void* workspace, size_t workspace_bytes, void* stream) {
    return decode_attn(s, plan_host, plan_dev, q, k_pages, v_pages, hidden_pages, W_K, W_V, W_packed, b_K, b_V,
                       block_tables, out, workspace, workspace_bytes, false, stream, nullptr, nullptr);
}

extern "C" int apt_hybrid_decode_attn_static(const apt_shape* s, const void* plan_host, void* plan_dev,
                                             const void* q, const void* k_pages, const void* v_pages, const void* hidden_pages,
                                             const void* W_K, const void* W_V, const void* W_packed,
                                             const void* b_K, const void* b_V, const int32_t* block_tables,
                                             void* out, void* stream) {
    return decode_attn(s, plan_host, plan_dev, q, k_pages, v_pages, hidden_pages, W_K, W_V, W_packed, b_K, b_V,
                       block_tables, out, nullptr, 0, true, stream, nullptr, nullptr);
}
