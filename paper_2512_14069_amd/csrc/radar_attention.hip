// Tree-verify attention for RADAR's target pass (Sec. 1: the draft tree is serialized
// and verified with masked attention in one LLM pass; Sec. 3), hand-written for
// gfx950: bf16 MFMA 32x32x16, 64-wide wavefronts, KV tiles staged through LDS.
//
// Work decomposition.  A workgroup (4 wavefronts) owns one (sequence, KV head,
// range of cache rows, block of up to 4 grouped query heads); wavefront w holds the
// T <= 64 tree rows of query head g = 4*block + w.  The cache rows [0, ctx_len +
// n_nodes) of a sequence are cut into splits of keys_per_split rows so that enough
// workgroups exist to pull from HBM on every CU; each split leaves an unnormalised
// partial (running max, sum, output) that a second small kernel merges.  K and V
// are read from HBM once per (split, query block), 16 bytes per lane, coalesced.
//
// Inside a wavefront everything is kept transposed: S^T = K Q^T (keys x queries)
// and O^T = V^T P^T (head-dim x queries).  With the MFMA accumulator layout a lane
// then owns ONE query column: its softmax statistics need no cross-lane traffic
// beyond one exchange with lane^32, the rescaling factor is lane-local, and the
// exponentiated scores already sit in the register order the next MFMA wants as
// its B operand (the key order inside a 16-key step is permuted consistently for
// P^T and V^T, which a contraction does not care about).
//
// The ancestor mask is never materialised in memory: each lane walks parents[]
// once for its query row and keeps the ancestor set as one 64-bit word; a tile
// that lies entirely in the prefix skips masking altogether.
#include "radar_device.h"

namespace radar {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = 4;
constexpr int kKT = 64;                    // cache rows per LDS tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;        // finite stand-in for "no score yet" (log2 units)

struct AttnArgs {
    const __bf16 *q, *k, *v;
    const int32_t *parents, *ctx_lens, *n_nodes;
    __bf16 *out;
    float *lse;
    int B, T, Hq, Hkv, G, S, kps, max_splits, n_qblk;
    int64_t q_sb, q_st, q_sh, kv_sb, kv_sh, kv_ss, o_sb, o_st, o_sh;
    float scale_log2;                      // softmax scale * log2(e)
    float *part_o;                         // [B][Hq][max_splits][D][64]
    float *part_ml;                        // [B][Hq][max_splits][2][64]
};

// byte offset of the 16-byte chunk `chunk` of cache row `key` in the K tile
template <int D>
__device__ __forceinline__ int ks_off(int key, int chunk) {
    return key * (D * 2) + ((chunk ^ (key & 7)) << 4);
}
// byte offset of element (d, pos) of the transposed V tile; pos = permuted key slot.
// 16-byte groups of a row are XOR-swizzled so that both the transposing writes
// (lanes differ in d/8) and the operand reads (lanes differ in d) spread over banks.
__device__ __forceinline__ int vt_off(int d, int pos) {
    const int f = (d ^ (d >> 3)) & 7;
    return d * (kKT * 2) + ((((pos >> 3) ^ f) & 7) << 4) + ((pos & 7) << 1);
}
// slot of key kappa (0..63) inside a tile: bits 2 and 3 swapped, so that the 8 values a
// lane holds in accumulator registers [8s, 8s+8) line up with MFMA k-slots [8*g2, 8*g2+8).
__device__ __forceinline__ int key_slot(int kappa) {
    return (kappa & ~12) | ((kappa & 4) << 1) | ((kappa & 8) >> 1);
}

template <int D, int NQB>
__global__ __launch_bounds__(kAttnThreads) void tree_attn_split_kernel(AttnArgs a) {
    constexpr int CH = D / 8;               // 16-byte chunks per cache row
    constexpr int KSTEPS = D / 16;          // MFMA k-steps of Q K^T
    constexpr int DB = D / 32;              // 32-row blocks of O^T
    constexpr int KLOADS = kKT * CH / kAttnThreads;     // 16-byte K loads per lane per tile
    constexpr int VKEYS = 4;                              // keys packed per transposed V write
    constexpr int VITEMS = CH * (kKT / VKEYS);            // (chunk, 4-key group) work items per tile
    constexpr int VPASSES = (VITEMS + kAttnThreads - 1) / kAttnThreads;
    static_assert(KLOADS >= 1 && kKT * CH % kAttnThreads == 0, "tile too small for 256 lanes");

    __shared__ __attribute__((aligned(16))) unsigned char Ks[kKT * D * 2];
    __shared__ __attribute__((aligned(16))) unsigned char Vt[D * kKT * 2];
    __shared__ int s_par[RADAR_T_MAX];

    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int sp = blockIdx.x;
    const int hk = blockIdx.y / a.n_qblk, qblk = blockIdx.y % a.n_qblk;
    const int b = blockIdx.z;
    const int L = a.ctx_lens[b];
    int nn = a.n_nodes ? a.n_nodes[b] : a.T;
    nn = max(1, min(nn, a.T));
    const int total = min(L + nn, a.S);                  // never read past the cache the caller described
    const int kbeg = sp * a.kps;
    if (L < 0 || kbeg >= total) return;
    const int kend = min(total, kbeg + a.kps);
    const int nsplit = (total + a.kps - 1) / a.kps;

    const int g = qblk * kAttnWaves + w;                  // query head within the group
    const bool active = g < a.G;
    const int h = hk * a.G + (active ? g : 0);
    const int j32 = lane & 31, g2 = lane >> 5;

    // ---- parents -> LDS, ancestor words (only if this split reaches the tree rows)
    if (tid < RADAR_T_MAX) s_par[tid] = (tid < nn) ? a.parents[(size_t)b * a.T + tid] : -1;
    __syncthreads();
    uint64_t anc[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        anc[qb] = 0;
        const int i = 32 * qb + j32;
        if (kend > L && i < nn) {
            uint64_t m = 1ull << i;
            int guard = i, p = s_par[i];
            while (p >= 0 && p < guard) { m |= 1ull << p; guard = p; p = s_par[p]; }
            anc[qb] = m;
        }
    }

    // ---- Q as MFMA B operands: lane (query j32 of block qb, half g2) holds d = 16*step + 8*g2 .. +8
    bf16x8 qreg[KSTEPS][NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        const int i = 32 * qb + j32;
        const __bf16 *qrow = a.q + (size_t)b * a.q_sb + (size_t)i * a.q_st + (size_t)h * a.q_sh;
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (active && i < a.T) raw = *reinterpret_cast<const uint4 *>(qrow + 16 * st + 8 * g2);
            qreg[st][qb] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    floatx16 oacc[DB][NQB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][qb][r] = 0.f;
    float m_run[NQB], l_run[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) { m_run[qb] = kNegBig; l_run[qb] = 0.f; }

    const __bf16 *kbase = a.k + (size_t)b * a.kv_sb + (size_t)hk * a.kv_sh;
    const __bf16 *vbase = a.v + (size_t)b * a.kv_sb + (size_t)hk * a.kv_sh;

    // global -> register staging of one tile
    uint4 kreg[KLOADS];
    uint4 vreg[VPASSES][VKEYS];
    auto load_tile = [&](int t0) {
#pragma unroll
        for (int i = 0; i < KLOADS; ++i) {
            const int c = i * kAttnThreads + tid;
            const int key = c / CH, ch = c % CH;
            const int kpos = t0 + key;
            kreg[i] = make_uint4(0, 0, 0, 0);
            if (kpos < kend) kreg[i] = *reinterpret_cast<const uint4 *>(kbase + (size_t)kpos * a.kv_ss + ch * 8);
        }
#pragma unroll
        for (int ps = 0; ps < VPASSES; ++ps) {
            const int item = ps * kAttnThreads + tid;
            const int ch = item % CH, kg = item / CH;
#pragma unroll
            for (int i = 0; i < VKEYS; ++i) {
                const int kpos = t0 + kg * VKEYS + i;
                vreg[ps][i] = make_uint4(0, 0, 0, 0);
                if (item < VITEMS && kpos < kend) vreg[ps][i] = *reinterpret_cast<const uint4 *>(vbase + (size_t)kpos * a.kv_ss + ch * 8);
            }
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < KLOADS; ++i) {
            const int c = i * kAttnThreads + tid;
            const int key = c / CH, ch = c % CH;
            *reinterpret_cast<uint4 *>(Ks + ks_off<D>(key, ch)) = kreg[i];
        }
#pragma unroll
        for (int ps = 0; ps < VPASSES; ++ps) {
            const int item = ps * kAttnThreads + tid;
            if (item >= VITEMS) break;
            const int ch = item % CH, kg = item / CH;
            const int pos0 = key_slot(kg * VKEYS);
            const uint32_t w0[4] = {vreg[ps][0].x, vreg[ps][0].y, vreg[ps][0].z, vreg[ps][0].w};
            const uint32_t w1[4] = {vreg[ps][1].x, vreg[ps][1].y, vreg[ps][1].z, vreg[ps][1].w};
            const uint32_t w2[4] = {vreg[ps][2].x, vreg[ps][2].y, vreg[ps][2].z, vreg[ps][2].w};
            const uint32_t w3[4] = {vreg[ps][3].x, vreg[ps][3].y, vreg[ps][3].z, vreg[ps][3].w};
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                // elements 2*e2 (low halves) and 2*e2+1 (high halves) of the four keys
                uint2 lo, hi;
                lo.x = (w0[e2] & 0xffffu) | (w1[e2] << 16);
                lo.y = (w2[e2] & 0xffffu) | (w3[e2] << 16);
                hi.x = (w0[e2] >> 16) | (w1[e2] & 0xffff0000u);
                hi.y = (w2[e2] >> 16) | (w3[e2] & 0xffff0000u);
                *reinterpret_cast<uint2 *>(Vt + vt_off(ch * 8 + 2 * e2, pos0)) = lo;
                *reinterpret_cast<uint2 *>(Vt + vt_off(ch * 8 + 2 * e2 + 1, pos0)) = hi;
            }
        }
    };

    const int ntiles = (kend - kbeg + kKT - 1) / kKT;
    load_tile(kbeg);
    for (int t = 0; t < ntiles; ++t) {
        const int t0 = kbeg + t * kKT;
        __syncthreads();                      // previous tile fully consumed
        store_tile();
        __syncthreads();
        if (t + 1 < ntiles) load_tile(t0 + kKT);   // in flight while this tile is computed
        if (!active) continue;

        const bool need_mask = (t0 + kKT > L) || (t0 + kKT > kend);
#pragma unroll
        for (int sub = 0; sub < kKT / 32; ++sub) {
            if (t0 + 32 * sub >= kend) break;
            // ---- S^T = K Q^T for 32 keys x (32*NQB) queries
            floatx16 sacc[NQB];
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[qb][r] = 0.f;
#pragma unroll
            for (int st = 0; st < KSTEPS; ++st) {
                const uint4 raw = *reinterpret_cast<const uint4 *>(Ks + ks_off<D>(32 * sub + j32, 2 * st + g2));
                const bf16x8 ka = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb)
                    sacc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[st][qb], sacc[qb], 0, 0, 0);
            }
            // ---- online softmax; register r of a lane is key 8*(r/4) + 4*g2 + r%4 of this sub-tile
            bf16x8 pk[NQB][2];
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) {
                float sv[16];
                float mx = kNegBig;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float sc = sacc[qb][r] * a.scale_log2;
                    if (need_mask) {
                        const int kpos = t0 + 32 * sub + 8 * (r >> 2) + 4 * g2 + (r & 3);
                        const int rel = kpos - L;
                        const bool ok = (kpos < kend) && (rel < 0 || ((anc[qb] >> (rel & 63)) & 1ull));
                        sc = ok ? sc : -INFINITY;
                    }
                    sv[r] = sc;
                    mx = fmaxf(mx, sc);
                }
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[qb], mx);
                const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_new);
                m_run[qb] = m_new;
                float rs = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = __builtin_amdgcn_exp2f(sv[r] - m_new);
                    rs += p;
                    pk[qb][r >> 3][r & 7] = (__bf16)p;
                }
                l_run[qb] = l_run[qb] * alpha + rs;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[db][qb][r] *= alpha;
            }
            // ---- O^T += V^T P^T
#pragma unroll
            for (int db = 0; db < DB; ++db) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const uint4 raw = *reinterpret_cast<const uint4 *>(Vt + vt_off(32 * db + j32, 32 * sub + 16 * s2 + 8 * g2));
                    const bf16x8 va = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
                    for (int qb = 0; qb < NQB; ++qb)
                        oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pk[qb][s2], oacc[db][qb], 0, 0, 0);
                }
            }
        }
    }
    if (!active) return;

    // ---- epilogue: a lane owns query i = 32*qb + j32; its registers hold d = 32*db + 8*(r/4) + 4*g2 + r%4
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        const int i = 32 * qb + j32;
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
        if (nsplit == 1) {
            if (i >= a.T) continue;
            __bf16 *orow = a.out + (size_t)b * a.o_sb + (size_t)i * a.o_st + (size_t)h * a.o_sh;
            const float inv = (i < nn && l_tot > 0.f) ? 1.0f / l_tot : 0.f;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                    bf16x4 o4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(i < nn ? oacc[db][qb][4 * r4 + e] * inv : 0.f);
                    *reinterpret_cast<bf16x4 *>(orow + 32 * db + 8 * r4 + 4 * g2) = o4;
                }
            if (a.lse && g2 == 0)
                a.lse[((size_t)b * a.T + i) * a.Hq + h] = (i < nn) ? (m_run[qb] + __builtin_amdgcn_logf(l_tot)) * kLn2 : 0.f;
        } else {
            const size_t unit = ((size_t)b * a.Hq + h) * a.max_splits + sp;
            float *po = a.part_o + unit * (size_t)(D * 64);
            float *pml = a.part_ml + unit * 128;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int d = 32 * db + 8 * (r >> 2) + 4 * g2 + (r & 3);
                    po[d * 64 + i] = oacc[db][qb][r];
                }
            if (g2 == 0) { pml[i] = m_run[qb]; pml[64 + i] = l_tot; }
        }
    }
}

// Merges the per-split partials of one (sequence, query head): 64 query rows x D.
template <int D>
__global__ __launch_bounds__(kAttnThreads) void tree_attn_merge_kernel(AttnArgs a) {
    const int h = blockIdx.x, b = blockIdx.y;
    const int L = a.ctx_lens[b];
    int nn = a.n_nodes ? a.n_nodes[b] : a.T;
    nn = max(1, min(nn, a.T));
    const int total = min(L + nn, a.S);
    const int nsplit = (total + a.kps - 1) / a.kps;
    if (L < 0 || nsplit <= 1) return;                       // the split kernel wrote the result itself

    const int i = threadIdx.x & 63, part = threadIdx.x >> 6; // query row, quarter of the head dim
    if (i >= a.T) return;
    const size_t unit0 = ((size_t)b * a.Hq + h) * a.max_splits;
    __bf16 *orow = a.out + (size_t)b * a.o_sb + (size_t)i * a.o_st + (size_t)h * a.o_sh;
    constexpr int DQ = D / 4;
    typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
    if (i >= nn) {
#pragma unroll
        for (int c = 0; c < DQ / 8; ++c) {
            bf16x8v z;
#pragma unroll
            for (int e = 0; e < 8; ++e) z[e] = (__bf16)0.f;
            *reinterpret_cast<bf16x8v *>(orow + part * DQ + 8 * c) = z;
        }
        if (a.lse && part == 0) a.lse[((size_t)b * a.T + i) * a.Hq + h] = 0.f;
        return;
    }
    float M = kNegBig;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, a.part_ml[(unit0 + s) * 128 + i]);
    float acc[DQ];
#pragma unroll
    for (int d = 0; d < DQ; ++d) acc[d] = 0.f;
    float lsum = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const float ms = a.part_ml[(unit0 + s) * 128 + i];
        const float ls = a.part_ml[(unit0 + s) * 128 + 64 + i];
        const float wgt = __builtin_amdgcn_exp2f(ms - M);
        lsum += wgt * ls;
        const float *po = a.part_o + (unit0 + s) * (size_t)(D * 64);
#pragma unroll
        for (int d = 0; d < DQ; ++d) acc[d] += wgt * po[(part * DQ + d) * 64 + i];
    }
    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
#pragma unroll
    for (int c = 0; c < DQ / 8; ++c) {
        bf16x8v o8;
#pragma unroll
        for (int e = 0; e < 8; ++e) o8[e] = (__bf16)(acc[8 * c + e] * inv);
        *reinterpret_cast<bf16x8v *>(orow + part * DQ + 8 * c) = o8;
    }
    if (a.lse && part == 0) a.lse[((size_t)b * a.T + i) * a.Hq + h] = (M + __builtin_amdgcn_logf(lsum)) * kLn2;
}

static int choose_keys_per_split(const radar_attn_desc *d) {
    if (d->keys_per_split > 0) return d->keys_per_split;
    const int G = d->Hq / d->Hkv;
    const int n_qblk = (G + kAttnWaves - 1) / kAttnWaves;
    const long units = (long)d->B * d->Hkv * n_qblk;
    const long target = 512;                                   // workgroups wanted for 256 CUs
    long ns = (target + units - 1) / units;
    if (ns < 1) ns = 1;
    long kps = ((long)d->S_max + ns - 1) / ns;
    kps = (kps + kKT - 1) / kKT * kKT;
    if (kps < 128) kps = 128;
    if (kps > 2048) kps = 2048;
    return (int)kps;
}

}  // namespace radar

using namespace radar;

static radar_status check_attn_desc(const radar_attn_desc *d) {
    if (!d) return RADAR_INVALID_ARG;
    if (d->B < 1 || d->T_max < 1 || d->Hq < 1 || d->Hkv < 1 || d->S_max < 1 || d->Hq % d->Hkv != 0)
        return RADAR_INVALID_ARG;
    if (d->keys_per_split < 0 || d->keys_per_split % kKT != 0) return RADAR_INVALID_ARG;
    if ((d->D != 64 && d->D != 128) || d->T_max > RADAR_T_MAX) return RADAR_UNSUPPORTED_SHAPE;
    if (d->B > 65535 || (long)d->Hkv * ((d->Hq / d->Hkv + 3) / 4) > 65535) return RADAR_UNSUPPORTED_SHAPE;
    return RADAR_OK;
}

extern "C" size_t radar_tree_attention_workspace_bytes(const radar_attn_desc *d) {
    if (check_attn_desc(d) != RADAR_OK) return 0;
    const int kps = choose_keys_per_split(d);
    const size_t max_splits = ((size_t)d->S_max + kps - 1) / kps;
    size_t bytes = 16384;
    if (max_splits > 1) bytes += (size_t)d->B * d->Hq * max_splits * ((size_t)d->D * 64 + 128) * sizeof(float);
    return (bytes + 255) & ~size_t(255);
}

extern "C" radar_status radar_tree_attention(const void *q, const void *k_cache, const void *v_cache,
                                             const int32_t *parents, const int32_t *ctx_lens, const int32_t *n_nodes,
                                             void *out, float *lse_out, const radar_attn_desc *d, void *workspace,
                                             size_t workspace_bytes, void *stream) {
    if (!q || !k_cache || !v_cache || !parents || !ctx_lens || !out || !workspace) return RADAR_INVALID_ARG;
    radar_status st = check_attn_desc(d);
    if (st != RADAR_OK) return st;
    if (workspace_bytes < radar_tree_attention_workspace_bytes(d)) return RADAR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return RADAR_INVALID_ARG;

    AttnArgs a;
    a.q = static_cast<const __bf16 *>(q); a.k = static_cast<const __bf16 *>(k_cache);
    a.v = static_cast<const __bf16 *>(v_cache);
    a.parents = parents; a.ctx_lens = ctx_lens; a.n_nodes = n_nodes;
    a.out = static_cast<__bf16 *>(out); a.lse = lse_out;
    a.B = d->B; a.T = d->T_max; a.Hq = d->Hq; a.Hkv = d->Hkv; a.G = d->Hq / d->Hkv; a.S = d->S_max;
    a.kps = choose_keys_per_split(d);
    a.max_splits = (d->S_max + a.kps - 1) / a.kps;
    a.n_qblk = (a.G + kAttnWaves - 1) / kAttnWaves;
    const int64_t D = d->D;
    a.q_sh = d->q_stride_h ? d->q_stride_h : D;
    a.q_st = d->q_stride_t ? d->q_stride_t : D * d->Hq;
    a.q_sb = d->q_stride_b ? d->q_stride_b : D * d->Hq * d->T_max;
    a.kv_ss = d->kv_stride_s ? d->kv_stride_s : D;
    a.kv_sh = d->kv_stride_h ? d->kv_stride_h : D * d->S_max;
    a.kv_sb = d->kv_stride_b ? d->kv_stride_b : D * d->S_max * d->Hkv;
    a.o_sh = d->out_stride_h ? d->out_stride_h : D;
    a.o_st = d->out_stride_t ? d->out_stride_t : D * d->Hq;
    a.o_sb = d->out_stride_b ? d->out_stride_b : D * d->Hq * d->T_max;
    // 16-byte alignment of every row the kernels touch with vector accesses
    const uintptr_t al = (uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out;
    const int64_t strides = a.q_sh | a.q_st | a.q_sb | a.kv_ss | a.kv_sh | a.kv_sb | a.o_sh | a.o_st | a.o_sb;
    if ((al & 15) != 0 || (strides & 7) != 0) return RADAR_INVALID_ARG;
    const float scale = d->softmax_scale != 0.f ? d->softmax_scale : 1.0f / sqrtf((float)d->D);
    a.scale_log2 = scale * kLog2e;
    char *ws = static_cast<char *>(workspace);
    a.part_o = reinterpret_cast<float *>(ws + 16384);
    a.part_ml = a.part_o + (size_t)d->B * d->Hq * a.max_splits * (size_t)(d->D * 64);

    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)a.max_splits, (unsigned)(a.Hkv * a.n_qblk), (unsigned)a.B), block(kAttnThreads);
    const bool narrow = d->T_max <= 32;
    if (d->D == 128) {
        if (narrow) hipLaunchKernelGGL((tree_attn_split_kernel<128, 1>), grid, block, 0, s, a);
        else        hipLaunchKernelGGL((tree_attn_split_kernel<128, 2>), grid, block, 0, s, a);
    } else {
        if (narrow) hipLaunchKernelGGL((tree_attn_split_kernel<64, 1>), grid, block, 0, s, a);
        else        hipLaunchKernelGGL((tree_attn_split_kernel<64, 2>), grid, block, 0, s, a);
    }
    if (hipGetLastError() != hipSuccess) return RADAR_HIP_ERROR;
    if (a.max_splits > 1) {
        const dim3 mgrid((unsigned)a.Hq, (unsigned)a.B);
        if (d->D == 128) hipLaunchKernelGGL(tree_attn_merge_kernel<128>, mgrid, block, 0, s, a);
        else             hipLaunchKernelGGL(tree_attn_merge_kernel<64>, mgrid, block, 0, s, a);
        if (hipGetLastError() != hipSuccess) return RADAR_HIP_ERROR;
    }
    return RADAR_OK;
}
