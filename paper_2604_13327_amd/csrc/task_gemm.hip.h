// Projection tile task: 16 weight rows x K against up to 64 activation columns, bf16 MFMA with
// fp32 accumulation (v_mfma_f32_16x16x32_bf16), weights streamed from HBM exactly once.
//
// Work split.  The 8 wavefronts of the workgroup split K; each streams its slice of all 16 rows
// with 16-byte non-temporal loads, keeping PF loads (PF KB per wave) in flight.  The first PF loads
// are issued BEFORE the task waits on its events (weight prefetch, paper Sec. 3.4 / 4.3), so HBM
// keeps streaming while the dependency resolves.  The activation operand (tiny, L2 resident) is
// fetched through a 2-deep register ring.  Partial tiles are reduced across waves through LDS in a
// fixed order (deterministic), then the epilogue runs on 8 x batch threads.
//
// The 16 rows of a tile are two groups of 8 (rowsA, rowsB): a RoPE tile takes rows i..i+7 and
// i+d/2..i+d/2+7 of one head (8 rotation pairs), a SwiGLU tile takes 8 gate rows and the 8 matching
// up rows, plain tiles take 16 consecutive rows.
#pragma once
#include "device_rt.hip.h"

namespace etc {

struct GemmTile {
    const uint16_t *rowsA, *rowsB;   // bf16 weights, first row of each 8-row group
    int ldw;                         // weight row stride (elements)
    int K;                           // reduction length, multiple of 256
    // activation operand: either fp32 rows normalised on the fly (RMSNorm prologue) ...
    const float *xf;
    const uint16_t *gain;
    float eps;
    int ldx;
    // ... or bf16 rows used as they are
    const uint16_t *xb;
    int ldxb;
    const int32_t *col_rows;         // optional gather: column n reads source row col_rows[n]
    int n_cols;                      // valid columns (batch rows or routed tokens), <= 16 * NB
};

constexpr uint16_t EPF_DUMP_LAYER = 0x8000;   // epilogue also records the layer's hidden state

enum EpiKind : int { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_STORE_F32 = 3, EPI_MOE_ACT = 4, EPI_MOE_Y = 5 };

struct Epilogue {
    int kind;
    int layer;
    uint16_t flags;
    int row0;                 // first output row (RESID / STORE), first f (SWIGLU), first pair index (QKV)
    int head;                 // QKV: global head index (q heads, then k heads, then v heads)
    const float *resid;       // RESID: [*, ld] fp32 added to the result
    float *outf;              // fp32 destination
    uint16_t *outb;           // bf16 destination
    int ld;                   // destination row stride
    int col0;                 // MoE: first destination row (permuted row of column 0)
};

constexpr int kRedFloats = kWaves * 4 * 64 * 4;   // cross-wave reduction buffer (32 KB)

__device__ __forceinline__ u32x4 load16_nt(const uint16_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}
__device__ __forceinline__ u32x4 load16(const uint16_t *p) { return *reinterpret_cast<const u32x4 *>(p); }

__device__ __forceinline__ void apply_epilogue(const Params &P, const Epilogue &e, int col, int mp, float lo, float hi);

// Waits of a projection task: wave-level.  per_wave: wave w waits on ev0 + w (its own K slice).
struct TaskWaits {
    int ev0, ev1, fn;
    bool per_wave;
};

template <int NB, bool NORM>
__device__ __forceinline__ bool gemm_tile_run(const Params &P, const GemmTile &g, const Epilogue &e, const TaskWaits &w,
                                           float *sm)
{
    const int wave = wave_id(), lane = lane_id();
    const int m = lane & 15, kg = lane >> 4;
    const int Kw = g.K / kWaves, n_it = Kw >> 5;
    const int kbase = wave * Kw + kg * 8;
    const uint16_t *wrow =
        (m < 8 ? g.rowsA + (size_t)m * (size_t)g.ldw : g.rowsB + (size_t)(m - 8) * (size_t)g.ldw) + kbase;

    // ---- weight prefetch: before the wait ------------------------------------------------
    constexpr int PF = 8;
    u32x4 wreg[PF];
#pragma unroll
    for (int j = 0; j < PF; ++j) {
        if (j < n_it) wreg[j] = load16_nt(wrow + j * 32);
        else wreg[j] = u32x4{0, 0, 0, 0};
    }

    // ---- E.wait() -------------------------------------------------------------------------
    // A wait that gives up records the error and the task still runs to completion (on stale
    // data): every wave keeps the same barrier sequence, so the kernel always drains.
    bool ok = wave_wait(P, w.per_wave ? w.ev0 + wave : w.ev0, w.fn);
    ok = wave_wait(P, w.ev1, w.fn) && ok;

    float *red = sm;
    float *rs = sm + kRedFloats;

    // ---- operand columns of this lane -------------------------------------------------------
    const float *xrow[NB];
    const uint16_t *brow[NB];
    float scale[NB];
    bool valid[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int col = nb * 16 + m;
        int row = col;
        valid[nb] = col < g.n_cols;
        if (valid[nb] && g.col_rows) row = g.col_rows[col];
        if (row < 0) valid[nb] = false;
        if (!valid[nb]) row = 0;
        xrow[nb] = NORM ? g.xf + (size_t)row * (size_t)g.ldx + kbase : nullptr;
        brow[nb] = NORM ? nullptr : g.xb + (size_t)row * (size_t)g.ldxb + kbase;
        scale[nb] = 0.f;
    }
    if (NORM) {   // RMSNorm prologue: 1 / sqrt(mean(x^2) + eps) of every operand row
        for (int col = wave; col < g.n_cols; col += kWaves) {
            int row = g.col_rows ? g.col_rows[col] : col;
            float s = 0.f;
            if (row >= 0) {
                const float *xr = g.xf + (size_t)row * (size_t)g.ldx;
                for (int i = lane * 4; i < g.K; i += 256) {
                    f32x4 v = *reinterpret_cast<const f32x4 *>(xr + i);
                    s += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
                }
            }
            s = wave_sum(s);
            if (lane == 0) rs[col] = 1.0f / sqrtf(s / (float)g.K + g.eps);
        }
        __syncthreads();
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) scale[nb] = valid[nb] ? rs[nb * 16 + m] : 0.f;
    }

    // ---- operand ring (depth 2) -------------------------------------------------------------
    struct Raw {
        f32x4 x0[NB], x1[NB];
        u32x4 gn;
        u32x4 b[NB];
    };
    Raw ring[2];
    auto fetch = [&](int s, Raw &r) {
        const int k = s * 32;
        if (NORM) {
            r.gn = load16(g.gain + kbase + k);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                if (valid[nb]) {
                    r.x0[nb] = *reinterpret_cast<const f32x4 *>(xrow[nb] + k);
                    r.x1[nb] = *reinterpret_cast<const f32x4 *>(xrow[nb] + k + 4);
                } else {
                    r.x0[nb] = f32x4{0, 0, 0, 0};
                    r.x1[nb] = f32x4{0, 0, 0, 0};
                }
            }
        } else {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) r.b[nb] = valid[nb] ? load16(brow[nb] + k) : u32x4{0, 0, 0, 0};
        }
    };
    auto operand = [&](const Raw &r, int nb) -> bf16x8 {
        u32x4 o;
        if (NORM) {
            const float sc = scale[nb];
            float g0 = bf16_bits_to_f32(r.gn.x & 0xFFFFu), g1 = bf16_bits_to_f32(r.gn.x >> 16);
            float g2 = bf16_bits_to_f32(r.gn.y & 0xFFFFu), g3 = bf16_bits_to_f32(r.gn.y >> 16);
            float g4 = bf16_bits_to_f32(r.gn.z & 0xFFFFu), g5 = bf16_bits_to_f32(r.gn.z >> 16);
            float g6 = bf16_bits_to_f32(r.gn.w & 0xFFFFu), g7 = bf16_bits_to_f32(r.gn.w >> 16);
            o.x = pack_bf16x2(r.x0[nb].x * sc * g0, r.x0[nb].y * sc * g1);
            o.y = pack_bf16x2(r.x0[nb].z * sc * g2, r.x0[nb].w * sc * g3);
            o.z = pack_bf16x2(r.x1[nb].x * sc * g4, r.x1[nb].y * sc * g5);
            o.w = pack_bf16x2(r.x1[nb].z * sc * g6, r.x1[nb].w * sc * g7);
        } else {
            o = r.b[nb];
        }
        return __builtin_bit_cast(bf16x8, o);
    };

    f32x4 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0, 0, 0, 0};

    fetch(0, ring[0]);
    if (n_it > 1) fetch(1, ring[1]);
    for (int it = 0; it < n_it; it += PF) {
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            const int s = it + j;
            if (s < n_it) {
                bf16x8 a = __builtin_bit_cast(bf16x8, wreg[j]);
                if (s + PF < n_it) wreg[j] = load16_nt(wrow + (s + PF) * 32);
                Raw &r = ring[j & 1];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, operand(r, nb), acc[nb], 0, 0, 0);
                if (s + 2 < n_it) fetch(s + 2, r);
            }
        }
    }

    // ---- cross-wave reduction (fixed order) and epilogue -------------------------------------
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
        *reinterpret_cast<f32x4 *>(red + ((size_t)(wave * NB + nb) * 64 + lane) * 4) = acc[nb];
    __syncthreads();
    for (int idx = threadIdx.x; idx < g.n_cols * 8; idx += kWgThreads) {
        const int col = idx >> 3, mp = idx & 7;
        const int nb = col >> 4, n = col & 15;
        float lo = 0.f, hi = 0.f;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) {
            const float *base = red + (size_t)(wv * NB + nb) * 256;
            lo += base[(n + 16 * (mp >> 2)) * 4 + (mp & 3)];
            hi += base[(n + 16 * ((mp + 8) >> 2)) * 4 + (mp & 3)];
        }
        apply_epilogue(P, e, col, mp, lo, hi);
    }
    return ok;
}

__device__ __forceinline__ bool gemm_tile_dispatch(const Params &P, const GemmTile &g, const Epilogue &e,
                                                   const TaskWaits &w, float *sm)
{
    const bool norm = g.xf != nullptr;
    if (g.n_cols <= 16) return norm ? gemm_tile_run<1, true>(P, g, e, w, sm) : gemm_tile_run<1, false>(P, g, e, w, sm);
    if (g.n_cols <= 32) return norm ? gemm_tile_run<2, true>(P, g, e, w, sm) : gemm_tile_run<2, false>(P, g, e, w, sm);
    return norm ? gemm_tile_run<4, true>(P, g, e, w, sm) : gemm_tile_run<4, false>(P, g, e, w, sm);
}

// cos / sin of the RoPE angle pos * theta^(-2i/d), evaluated in double (exact range reduction for
// positions in the thousands); kept out of line: it is called by 8 x batch threads per tile only.
__device__ __noinline__ void rope_cos_sin(int pos, int i, int d, float theta, float *cs, float *sn)
{
    const double inv = pow((double)theta, -2.0 * (double)i / (double)d);
    double s, c;
    sincos((double)pos * inv, &s, &c);
    *cs = (float)c;
    *sn = (float)s;
}

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

__device__ __forceinline__ void apply_epilogue(const Params &P, const Epilogue &e, int col, int mp, float lo, float hi)
{
    switch (e.kind) {
    case EPI_QKV: {
        const int b = col, half = P.d >> 1, i = e.row0 + mp;
        const int pos = P.kv_len[b];
        float a = lo, c = hi;
        if (e.head < P.nq + P.nkv) {   // q and k heads are rotated to position pos
            float cs, sn;
            rope_cos_sin(pos, i, P.d, P.theta, &cs, &sn);
            a = lo * cs - hi * sn;
            c = lo * sn + hi * cs;
        }
        if (e.head < P.nq) {
            float *q = P.qbuf + (size_t)b * (size_t)(P.nq * P.d) + (size_t)e.head * P.d;
            q[i] = a;
            q[i + half] = c;
        } else {
            const bool is_k = e.head < P.nq + P.nkv;
            const int kvh = is_k ? e.head - P.nq : e.head - P.nq - P.nkv;
            const int page = P.page_ids[P.page_indptr[b] + pos / P.page];
            const size_t off = (size_t)e.layer * (size_t)P.pool_layer_stride +
                               (((size_t)page * P.page + (size_t)(pos % P.page)) * P.nkv + kvh) * (size_t)P.d;
            uint16_t *dst = (is_k ? P.kpool : P.vpool) + off;
            dst[i] = f32_to_bf16_bits(a);
            dst[i + half] = f32_to_bf16_bits(c);
        }
        break;
    }
    case EPI_RESID: {
        const int b = col;
        const size_t o0 = (size_t)b * e.ld + e.row0 + mp, o1 = o0 + 8;
        const float v0 = e.resid[o0] + lo, v1 = e.resid[o1] + hi;
        e.outf[o0] = v0;
        e.outf[o1] = v1;
        if (e.flags & TF_LAST_LAYER) {
            P.hidden_out[o0] = f32_to_bf16_bits(v0);
            P.hidden_out[o1] = f32_to_bf16_bits(v1);
        }
        if (e.flags & EPF_DUMP_LAYER) {
            float *dbg = P.layer_hidden + (size_t)e.layer * (size_t)kMaxBatch * e.ld;
            dbg[o0] = v0;
            dbg[o1] = v1;
        }
        break;
    }
    case EPI_SWIGLU: {
        e.outb[(size_t)col * e.ld + e.row0 + mp] = f32_to_bf16_bits(silu_f(lo) * hi);
        break;
    }
    case EPI_STORE_F32: {
        e.outf[(size_t)col * e.ld + e.row0 + mp] = lo;
        e.outf[(size_t)col * e.ld + e.row0 + mp + 8] = hi;
        break;
    }
    case EPI_MOE_ACT: {
        e.outb[(size_t)(e.col0 + col) * e.ld + e.row0 + mp] = f32_to_bf16_bits(silu_f(lo) * hi);
        break;
    }
    case EPI_MOE_Y: {
        e.outf[(size_t)(e.col0 + col) * e.ld + e.row0 + mp] = lo;
        e.outf[(size_t)(e.col0 + col) * e.ld + e.row0 + mp + 8] = hi;
        break;
    }
    }
}

}  // namespace etc
