// Tree-verify attention for RADAR's target pass (Sec. 1: the draft tree is serialized
// and verified with masked attention in one LLM pass; Sec. 3), hand-written for
// gfx950: bf16 MFMA 32x32x16, 64-wide wavefronts, KV tiles staged through LDS.
//
// Inside a wavefront everything is kept transposed: S^T = K Q^T (keys x queries)
// and O^T = V^T P^T (head-dim x queries).  With the MFMA accumulator layout a lane
// then owns ONE query column: its softmax statistics need no cross-lane traffic
// beyond one exchange with lane^32, the rescaling factor is lane-local, and the
// exponentiated scores already sit in the register order the next MFMA wants as
// its B operand (the key order inside a 16-key step is permuted consistently for
// P^T and V^T, which a contraction does not care about).  The running output is
// rescaled only when some lane's maximum actually moved.
//
// The ancestor mask is never materialised in memory: each lane walks parents[]
// once for its query row and keeps the ancestor set as one 64-bit word; a tile
// that lies entirely in the prefix skips masking altogether.
//
// Work decomposition.  A workgroup of eight wavefronts owns (sequence, KV head,
// range of cache rows, block of eight (query head, 32 tree rows) units); each
// wavefront is one unit, and all eight share every K/V tile through LDS, so KV
// comes from HBM once per group of heads.  Two wavefronts per SIMD let one
// wavefront's MFMAs run underneath the other's softmax arithmetic.  Tiles are
// double-buffered in LDS (one barrier per tile) and the next tile's global loads
// are in flight during the arithmetic.  Ranges of cache rows are merged from partials
// (fp16 pairs scaled per row, plus maximum, sum and scale in fp32) by a small second kernel; how many ranges to cut is decided on the host
// from a cost model that counts whole rounds of resident workgroups and the
// partial traffic.
#include "radar_device.h"
#include <type_traits>
#include "radar_host.h"

namespace radar {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));     // a 16-byte load/store unit kept in registers

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
    int B, T, Hq, Hkv, G, S, kps, max_splits, n_ublk, nqb;   // nqb 32-row blocks per head, n_ublk workgroups per KV range
    int64_t q_sb, q_st, q_sh, kv_sb, kv_sh, kv_ss, o_sb, o_st, o_sh;
    float scale_log2;                      // softmax scale * log2(e), > 0
    uint32_t *part_o;                      // [B][Hq][max_splits][D/2][64]: partial outputs, fp16 pairs (d, d+1), scaled per row
    float *part_ml;                        // [B][Hq][max_splits][3][64]: running maximum (log2 units), sum, and the scale of part_o
};

// Byte offset of the 16-byte chunk `chunk` of cache row `key` in a K tile.  The chunks of a row are
// XOR-swizzled with the row number so that the sixteen lanes of one pass of a 16-byte operand read
// (sixteen consecutive rows, the same chunk) cover all 64 banks: 16 distinct chunk slots at D = 128
// (256-byte rows), 8 slots times the two rows of a 256-byte bank period at D = 64.
template <int D>
__device__ __forceinline__ int ks_off(int key, int chunk) {
    constexpr int CH = D / 8;
    return key * (D * 2) + ((chunk ^ ((key >> (CH == 16 ? 0 : 1)) & (CH - 1))) << 4);
}
// byte offset of element (d, pos) of a transposed V tile; pos = permuted key slot.
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

// byte offset of 16-byte chunk `chunk` of row `row` in a row-major V tile that is read by transposing
// LDS reads: one pass of such a read (32 lanes) touches 64 consecutive bytes of four consecutive rows,
// and with 256-byte rows these would meet in the same banks; the row's two low bits move its 64-byte
// windows apart.  (8 rows + 8 keeps the swizzle: the second read of a pair differs by a constant.)
template <int D>
__device__ __forceinline__ int vs_off(int row, int chunk) {
    static_assert(D == 128, "row-major V tiles are built for 256-byte rows");
    return row * (D * 2) + ((chunk ^ ((row & 3) << 2)) << 4);
}

// v = keep ? v : 0 without a branch (a select after a load tempts the compiler into a
// conditional load, and conditional loads into register arrays wreck register allocation)
__device__ __forceinline__ void and_mask(u32x4 &v, bool keep) {
    v &= 0u - (uint32_t)keep;
}

// Ancestor word of tree row i (bit a set <=> a is i or an ancestor of i).  par[] holds the
// sequence's parents in LDS.  Terminates and stays in bounds for any content: the chain is
// followed only while it strictly decreases.
__device__ __forceinline__ uint64_t ancestor_word(const int *par, int i) {
    uint64_t m = 1ull << i;
    int guard = i, p = par[i];
    while (p >= 0 && p < guard) { m |= 1ull << p; guard = p; p = par[p];}
    return m;
}

// One wavefront, one 64-row tile that sits in LDS, in three phases: scores into
// `sacc` (register r of sub-tile `sub` is row 32*sub + 8*(r/4) + 4*g2 + r%4), masked online softmax
// from `sacc` into the bf16 operand `pk` (rescaling the output accumulators when the maximum moved),
// and the update of the transposed output accumulators, from a transposed V tile (vt_off) or, with
// VTR, from a row-major one (vs_off) through transposing LDS reads.
// The lane's query operands are passed in registers (qop: row j32 of the block, d = 16*st + 8*g2
// .. +8; 32 VGPRs at D = 128): every LDS byte not read matters here, the eight wavefronts of a
// workgroup already read each K and V tile eight times over.  K operands are read from LDS four
// MFMAs before they are needed and the two score sub-tiles (the four output blocks) take turns, so
// that consecutive MFMAs are independent and none starts by waiting for LDS.
//   t0        cache row of the tile's first key;  L = prefix length;  kend = end of this range
//   first     true if the accumulators are still zero (no rescaling needed)
typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef const __attribute__((address_space(3))) u32x4 *lds_u32x4;

// kaddr(k): where step k's K operand sits in LDS (sub-tile k % 2, 16-byte chunk 2 * (k / 2) + g2 of row j32)
template <int D, typename KAddr>
__device__ __forceinline__ void tile_scores(KAddr kaddr, const bf16x8 (&qop)[D / 16], floatx16 (&sacc)[2]) {
    constexpr int KSTEPS = D / 16, NS = 2 * KSTEPS, kAhead = 4;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[sub][r] = 0.f;
    auto kread = [&](int k) { return *kaddr(k); };
    u32x4 kf[kAhead];
#pragma unroll
    for (int k = 0; k < kAhead; ++k) kf[k] = kread(k);
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        const u32x4 cur = kf[k % kAhead];
        if (k + kAhead < NS) kf[k % kAhead] = kread(k + kAhead);
        sacc[k & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cur), qop[k >> 1], sacc[k & 1], 0, 0, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);          // the order written above, for the scheduler
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (k + kAhead < NS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
}

template <int D>
__device__ __forceinline__ void tile_softmax(floatx16 (&sacc)[2], floatx16 (&oacc)[D / 32][1], float &m_run, float &l_run,
                                           uint64_t anc, int t0, int L, int kend, bool first, float scale_log2,
                                           bf16x8 (&pk)[2][2]) {
    constexpr int DB = D / 32;
    const int g2 = lane_id() >> 5;
    if ((t0 + kKT > L) || (t0 + kKT > kend)) {                       // wave-uniform; prefix tiles skip it
        const int pre = L - t0;                                      // prefix keys in this tile (may be <= 0 or >= 64)
        uint64_t allow = pre >= 64 ? ~0ull : (pre > 0 ? ((1ull << pre) - 1) : 0ull);
        if (pre > -64 && pre < 64) allow |= pre >= 0 ? (anc << pre) : (anc >> (-pre));
        const int len = kend - t0;
        if (len < 64) allow &= len > 0 ? ((1ull << len) - 1) : 0ull;
        allow >>= 4 * g2;
        const uint32_t aw[2] = {(uint32_t)allow, (uint32_t)(allow >> 32)};
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                sacc[sub][r] = ((aw[sub] >> (8 * (r >> 2) + (r & 3))) & 1u) ? sacc[sub][r] : -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[sub][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx * scale_log2);               // scale_log2 > 0; -inf stays -inf
    if (!first) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
        if (__any(alpha != 1.0f)) {                                  // wave-uniform: most tiles skip this
#pragma unroll
            for (int db = 0; db < DB; ++db) {
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][0][r] *= alpha;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    m_run = m_new;
    float rs = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[sub][r], scale_log2, -m_new));
            rs += p;
            pk[sub][r >> 3][r & 7] = (__bf16)p;
        }
    l_run += rs;
}

// vaddr(k, hi): VTR = false: where step k's V^T operand sits (16 bytes; hi unused); VTR = true: the 8-byte
// piece this lane names for the first (hi = 0) or second (hi = 1) transposing read of step k
template <int D, bool VTR, typename VAddr>
__device__ __forceinline__ void tile_pv(VAddr vaddr, const bf16x8 (&pk)[2][2], floatx16 (&oacc)[D / 32][1]) {
    constexpr int DB = D / 32, NP = 4 * DB, kAhead = 4;
    // V^T operand straight from the row-major tile, by two transposing LDS reads.  In each block of 16
    // lanes, lane 4j+q names an 8-byte piece (row kv0+j, elements 4q..4q+3 of the block's 16) and lane l
    // receives element l%4 of the pieces named by lanes 4j + l/4, j = 0..3: its own d for four
    // consecutive rows.  Rows 16ss + 4g2 .. +4 fill k-slots 8g2 .. 8g2+3 and the rows eight further on
    // fill 8g2+4 .. 8g2+7, which is where the P operand has them.
    typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
    typedef bf16x4_t __attribute__((address_space(3))) *lds_b64;
    auto vread = [&](int k) {
        if constexpr (!VTR) {
            return __builtin_bit_cast(bf16x8, *(lds_u32x4)vaddr(k, 0));
        } else {
            const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64)vaddr(k, 0));
            const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64)vaddr(k, 1));
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    bf16x8 vf[kAhead];
#pragma unroll
    for (int k = 0; k < kAhead; ++k) vf[k] = vread(k);
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const bf16x8 cur = vf[k % kAhead];
        if (k + kAhead < NP) vf[k % kAhead] = vread(k + kAhead);
        const int db = k % DB, ss = k / DB;
        oacc[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, pk[ss >> 1][ss & 1], oacc[db][0], 0, 0, 0);
    }
}

// ===================================================================== group-share kernel
// 512 lanes: eight wavefronts, two per SIMD, so that one wavefront's MFMAs run underneath the
// other's softmax arithmetic.  A wavefront is one (query head, block of 32 tree rows); the eight of
// a workgroup share every K/V tile through LDS.
constexpr int kGsThreads = 512;
constexpr int kGsWaves = kGsThreads / kWave;

// Staging of one 64-row K/V tile by the 512 lanes of the workgroup, no request made twice and the
// same work for every wavefront (a wavefront that staged more than the others would reach the tile's
// barrier after them, and everybody would wait for it): every lane fetches 16-byte chunks of K rows
// (two at D = 128) and one V item = one chunk of two consecutive cache rows, which it interleaves
// into the transposed tile with 4-byte LDS writes.  Branch-free loads: rows past the range re-read
// the last valid row; V is zeroed on its way into LDS (0 * anything must stay 0; masking right
// after the load would make the wavefront wait for its own loads), K is masked by the softmax.
template <int D>
struct GsTileRegs {
    static constexpr int CH = D / 8;                                       // 16-byte chunks per row
    static constexpr int KL = kKT * CH / 512;                              // K chunks per lane: 2 at D = 128, 1 at D = 64
    static constexpr int VITEMS = CH * (kKT / 2);                          // (chunk, row pair) items: 512 at D = 128, 256 at D = 64
    u32x4 k[KL], v[2];
};

// (One straight line of loads, no separate path for tiles that need no clamping: wherever loads sit
// under a condition the compiler cannot tell how many are in flight at the store, and waits for all
// of them, the tile after next included.)
template <int D>
__device__ __forceinline__ void gs_load_tile(GsTileRegs<D> &g, const __bf16 *kbase, const __bf16 *vbase, int kv_ss,
                                             int t0, int kend, int tid) {
    constexpr int CH = GsTileRegs<D>::CH;
    const int item = min(tid, GsTileRegs<D>::VITEMS - 1);
    const int ch = item % CH, kp = item / CH;
#pragma unroll
    for (int i = 0; i < GsTileRegs<D>::KL; ++i) {
        const int c = i * 512 + tid;
        const int kpos = min(t0 + c / CH, kend - 1);
        g.k[i] = *reinterpret_cast<const u32x4 *>(kbase + (uint32_t)(kpos * kv_ss + (c % CH) * 8));
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int kpos = min(t0 + 2 * kp + i, kend - 1);
        g.v[i] = *reinterpret_cast<const u32x4 *>(vbase + (uint32_t)(kpos * kv_ss + ch * 8));
    }
}

// t0, kend: the tile's first cache row and the end of the range, as given to gs_load_tile
template <int D>
__device__ __forceinline__ void gs_store_tile(const GsTileRegs<D> &g, unsigned char *Ks, unsigned char *Vt, int t0, int kend,
                                              int tid) {
    constexpr int CH = GsTileRegs<D>::CH;
#pragma unroll
    for (int i = 0; i < GsTileRegs<D>::KL; ++i) {
        const int c = i * 512 + tid;
        *reinterpret_cast<u32x4 *>(Ks + ks_off<D>(c / CH, c % CH)) = g.k[i];
    }
    if (tid < GsTileRegs<D>::VITEMS) {
        const int ch = tid % CH, kp = tid / CH;
        u32x4 v0 = g.v[0], v1 = g.v[1];
        if (t0 + kKT > kend) {                                             // wave-uniform: a range's last tile only
            and_mask(v0, t0 + 2 * kp < kend);
            and_mask(v1, t0 + 2 * kp + 1 < kend);
        }
        const int pos0 = key_slot(2 * kp);                                 // even; the pair's second row sits next to it
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            // elements 2*e2 (low halves) and 2*e2+1 (high halves) of the two rows
            const uint32_t lo = (v0[e2] & 0xffffu) | (v1[e2] << 16);
            const uint32_t hi = (v0[e2] >> 16) | (v1[e2] & 0xffff0000u);
            *reinterpret_cast<uint32_t *>(Vt + vt_off(ch * 8 + 2 * e2, pos0)) = lo;
            *reinterpret_cast<uint32_t *>(Vt + vt_off(ch * 8 + 2 * e2 + 1, pos0)) = hi;
        }
    }
}

// End of a group-share kernel: a lane owns query i; its accumulator registers O(db, r) hold
// d = 32*db + 8*(r/4) + 4*g2 + r%4 of the transposed output.
template <int D, typename Acc>
__device__ __forceinline__ void gs_finish(const AttnArgs &a, Acc O, float m_run, float l_run, int b, int h, int i, int nn,
                                          int sp, int nsplit) {
    constexpr int DB = D / 32;
    const int g2 = lane_id() >> 5;
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (nsplit == 1) {
        if (i >= a.T) return;
        __bf16 *orow = a.out + (size_t)b * a.o_sb + (size_t)i * a.o_st + (size_t)h * a.o_sh;
        const float inv = (i < nn && l_tot > 0.f) ? 1.0f / l_tot : 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                bf16x4 o4;
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(i < nn ? O(db, 4 * r4 + e) * inv : 0.f);
                *reinterpret_cast<bf16x4 *>(orow + 32 * db + 8 * r4 + 4 * g2) = o4;
            }
        if (a.lse && g2 == 0)
            a.lse[((size_t)b * a.T + i) * a.Hq + h] = (i < nn) ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : 0.f;
    } else {
        // Partial result of this key range: the row's output normalised by its own l and by the row's
        // largest magnitude, as fp16 pairs (d, d+1) -- [D/2][64 rows] words, so that 32 lanes still write
        // 128 contiguous bytes -- plus (m, l, magnitude) in fp32.  The partials of all ranges together
        // outweigh the K/V bytes, and writing them is what the tail of this kernel waits for; halving
        // them costs 2^-11 of the row's largest element in precision, an eighth of the bf16 rounding of
        // the final output.  Written through: nothing is left dirty in L2 for the end of the kernel.
        const size_t unit = ((size_t)b * a.Hq + h) * a.max_splits + sp;
        uint32_t *po = a.part_o + unit * (size_t)(D / 2 * 64);
        float *pml = a.part_ml + unit * 192;
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        float amax = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) amax = fmaxf(amax, fabsf(O(db, r)));
        amax = fmaxf(amax, __shfl_xor(amax, 32)) * inv;          // both halves of the row's d range
        const float mag = amax > 0.f && amax < 3.0e38f ? amax : 1.f;
        const float scl = inv / mag;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int rp = 0; rp < 8; ++rp) {
                const int r = 2 * rp;
                const int d = 32 * db + 8 * (r >> 2) + 4 * g2 + (r & 3);
                const _Float16 lo = (_Float16)(O(db, r) * scl), hi = (_Float16)(O(db, r + 1) * scl);
                const uint32_t word = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
                store_shared_result(&po[(d >> 1) * 64 + i], word);
            }
        if (g2 == 0) {
            store_shared_result(&pml[i], m_run);
            store_shared_result(&pml[64 + i], l_tot);
            store_shared_result(&pml[128 + i], mag);
        }
    }
}

template <int D, bool DEEP>
__global__ __launch_bounds__(kGsThreads) void tree_attn_gs_kernel(AttnArgs a) {
    constexpr int DB = D / 32;              // 32-row blocks of O^T

    constexpr int TILE = 2 * kKT * D * 2;   // one K tile ([64][D] bf16, swizzled) + one V^T tile ([D][64], swizzled)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int *s_par = reinterpret_cast<int *>(smem + 2 * TILE);

    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int sp = blockIdx.x;
    // The blocks of units that share a range of cache rows are ranges x KV heads apart in workgroup number:
    // a multiple of eight with eight KV heads, and consecutive numbers go to consecutive XCDs, so the
    // blocks meet in one XCD's L2 and their rows come from HBM once.
    const int hk = blockIdx.y, ublk = blockIdx.z % a.n_ublk;
    const int b = blockIdx.z / a.n_ublk;
    const int kbeg = sp * a.kps;                          // < S: the grid has ceil(S / kps) ranges

    const int u = ublk * kGsWaves + w;                    // (head within the group, block of 32 rows)
    const int g = u / a.nqb, qb = u % a.nqb;
    const bool active = g < a.G;
    const int h = hk * a.G + (active ? g : 0);
    const int j32 = lane & 31, g2 = lane >> 5;
    const int i = 32 * qb + j32;                          // this lane's tree row

    const __bf16 *kbase = a.k + (size_t)b * a.kv_sb + (size_t)hk * a.kv_sh;
    const __bf16 *vbase = a.v + (size_t)b * a.kv_sb + (size_t)hk * a.kv_sh;
    const int kv_ss = (int)a.kv_ss;          // 32-bit offsets inside one head's cache (checked on the host)

    // The first tile and the query rows are requested before the sequence's context length and tree size
    // are known (two dependent scalar loads, most of a microsecond in a cold start): rows are clamped to
    // the cache the caller described instead of to the end of the range.  Whatever rows past that end
    // hold is never used: their scores are masked by selection and their V rows zeroed on the way into
    // LDS, both from the range's real end below.
    // DEEP (ranges of many tiles): staging runs two tiles ahead through two register sets, which hides
    // HBM latency better but doubles the loop's code; short ranges keep the compact one-ahead loop
    // (their time goes into a cold start, where code size counts).
    GsTileRegs<D> regs0, regs1;
    gs_load_tile<D>(regs0, kbase, vbase, kv_ss, kbeg, a.S, tid);
    // this lane's query operands, kept in registers for the whole kernel: row i, d = 16*st + 8*g2 .. +8
    bf16x8 qop[D / 16];
    {
        const __bf16 *qrow = a.q + (size_t)b * a.q_sb + (size_t)h * a.q_sh + (uint32_t)(min(i, a.T - 1) * (int)a.q_st);
#pragma unroll
        for (int st = 0; st < D / 16; ++st) {
            u32x4 raw = *reinterpret_cast<const u32x4 *>(qrow + 16 * st + 8 * g2);
            and_mask(raw, active && i < a.T);
            qop[st] = __builtin_bit_cast(bf16x8, raw);
        }
    }
    const int L = a.ctx_lens[b];
    int nn = a.n_nodes ? a.n_nodes[b] : a.T;
    nn = max(1, min(nn, a.T));
    const int total = min(L + nn, a.S);                  // never read past the cache the caller described
    if (L < 0 || kbeg >= total) return;
    const int kend = min(total, kbeg + a.kps);
    const int nsplit = (total + a.kps - 1) / a.kps;
    const int ntiles = (kend - kbeg + kKT - 1) / kKT;
    if (DEEP) gs_load_tile<D>(regs1, kbase, vbase, kv_ss, kbeg + kKT, kend, tid);
    if (tid < RADAR_T_MAX) s_par[tid] = a.parents[(size_t)b * a.T + min(tid, nn - 1)];
    gs_store_tile<D>(regs0, smem, smem + TILE / 2, kbeg, kend, tid);
    __syncthreads();
    if (DEEP) gs_load_tile<D>(regs0, kbase, vbase, kv_ss, kbeg + 2 * kKT, kend, tid);
    else if (ntiles > 1) gs_load_tile<D>(regs0, kbase, vbase, kv_ss, kbeg + kKT, kend, tid);
    uint64_t anc[1];
    anc[0] = (kend > L && i < nn) ? ancestor_word(s_par, i) : 0ull;

    floatx16 oacc[DB][1];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][0][r] = 0.f;
    float m_run[1] = {kNegBig}, l_run[1] = {0.f};

    // Two tile buffers in LDS: while tile t is consumed from one, every wavefront drops its share of
    // tile t+1 into the other as soon as it is done with t.  One barrier per tile: it publishes tile
    // t+1 and tells that nobody reads tile t any more.
    auto step = [&](int t, GsTileRegs<D> &next_regs, int ahead) {
        unsigned char *cur = smem + (t & 1) * TILE, *nxt = smem + ((t + 1) & 1) * TILE;
        if (active) {
            floatx16 sacc[2];
            bf16x8 pk[2][2];
            const unsigned char *Vt = cur + TILE / 2;
            tile_scores<D>([&](int k) { return (lds_u32x4)(cur + ks_off<D>(32 * (k & 1) + j32, 2 * (k >> 1) + g2)); }, qop, sacc);
            tile_softmax<D>(sacc, oacc, m_run[0], l_run[0], anc[0], kbeg + t * kKT, L, kend, t == 0, a.scale_log2, pk);
            tile_pv<D, false>([&](int k, int) { return (const lds_byte *)(Vt + vt_off(32 * (k % DB) + j32, 16 * (k / DB) + 8 * g2)); },
                              pk, oacc);
        }
        if (t + 1 < ntiles) {
            gs_store_tile<D>(next_regs, nxt, nxt + TILE / 2, kbeg + (t + 1) * kKT, kend, tid);
            __syncthreads();
        }
        // Two tiles ahead, the loads are issued whether or not the range still has such a tile (rows past
        // its end re-read its last row): only if every step issues the same loads does the compiler
        // know how many are in flight when a set is stored, and wait for that set alone.
        if (DEEP || t + ahead < ntiles) gs_load_tile<D>(next_regs, kbase, vbase, kv_ss, kbeg + (t + ahead) * kKT, kend, tid);
    };
    if (DEEP) {                                           // unrolled by two: odd tiles travel through regs1, even ones through regs0
        int t = 0;
        for (; t + 1 < ntiles; t += 2) {
            step(t, regs1, 3);
            step(t + 1, regs0, 3);
        }
        if (t < ntiles) step(t, regs1, 3);
    } else {
        for (int t = 0; t < ntiles; ++t) step(t, regs0, 2);
    }
    if (!active) return;
    gs_finish<D>(a, [&](int db, int r) { return oacc[db][0][r]; }, m_run[0], l_run[0], b, h, i, nn, sp, nsplit);
}

// ===================================================================== group-share kernel, long ranges
// The same decomposition with tiles that reach LDS without passing through registers: every wavefront
// issues four loads per tile that write LDS directly (1 KB each: four rows of K or V; a lane's 16 bytes
// land at the instruction's LDS base + 16 * lane, so the swizzle is applied by choosing which chunk of
// the row the lane fetches), a pair of tiles ahead of the pair being consumed, four tile buffers.  V
// stays row-major and is transposed by the LDS reads that fetch the operands.  No staging registers,
// no vector instructions for the transposition, one barrier per pair of tiles.  Rows past the end
// of a range re-read its last row: their scores are masked, and the row they repeat is a cache row
// whose values the result depends on anyway (0 * finite = 0).
constexpr int kLdBufs = 4;

// A lane's share of a tile: two chunks of K and two of V.  Wavefront w loads the row groups 2w and
// 2w + 1 (four rows, 1 KB each); the lane's 16 bytes land at the group's LDS base + 16 * lane, i.e. in
// slot lane % 16 of row 4 * group + lane / 16, so it fetches the chunk that the swizzle puts there.
// The byte offsets inside a tile are fixed for the kernel's lifetime.
struct LdLane {
    uint32_t offk[2], offv[2];        // from the tile's first row, rows kv_ss elements apart
};

template <int D>
__device__ __forceinline__ LdLane ld_lane_offsets(int kv_ss, int w, int lane) {
    static_assert(D == 128, "1 KB per instruction = four 256-byte rows");
    LdLane o;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = 4 * (2 * w + i) + (lane >> 4), slot = lane & 15;
        o.offk[i] = (uint32_t)(row * kv_ss) * 2 + (uint32_t)((slot ^ (row & 15)) << 4);          // inverse of ks_off's swizzle
        o.offv[i] = (uint32_t)(row * kv_ss) * 2 + (uint32_t)((slot ^ ((row & 3) << 2)) << 4);    // inverse of vs_off's
    }
    return o;
}

// Issues this wavefront's four loads of the tile whose first cache row is t0 into the buffer `buf`.
// Issued as assembly: told about loads that write LDS, the compiler waits for all of them before the
// next LDS read it cannot tell apart from their targets, which would undo the run-ahead; the waits for
// these loads are the explicit ones in the kernel's loop.  (m0 is a reserved register: the compiler
// sets it right before each of its own uses and warns about the clobber.)  A tile inside the range
// takes a scalar base and the lane's fixed offsets, no vector arithmetic; a tile that reaches past the
// end of the range clamps every row to the range's last one.
template <int D>
__device__ __forceinline__ void ld_issue_tile(unsigned char *buf, const __bf16 *kbase, const __bf16 *vbase, int kv_ss, int t0,
                                              int kend, int w, int lane, const LdLane &o) {
    // (the wavefront's number is the same in every lane, which the compiler cannot see: the LDS bases below have to be scalars)
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)buf + (uint32_t)w * 2048);
    if (t0 + kKT <= kend) {                                          // wave-uniform
        // (the tile bases are the same in every lane; passed through readfirstlane so that they are scalars
        // for the assembly below whatever the compiler knows about their uniformity)
        auto scalar_ptr = [](const __bf16 *p) {
            const uint64_t v = (uint64_t)(uintptr_t)p;
            const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
            return (const __bf16 *)(uintptr_t)(((uint64_t)hi << 32) | lo);
        };
        const __bf16 *kt = scalar_ptr(kbase + (uint32_t)(t0 * kv_ss)), *vt = scalar_ptr(vbase + (uint32_t)(t0 * kv_ss));
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t ldsk = lds0 + i * 1024, ldsv = ldsk + kKT * D * 2;
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(ldsk), "v"(o.offk[i]), "s"(kt) : "memory", "m0");
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(ldsv), "v"(o.offv[i]), "s"(vt) : "memory", "m0");
        }
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = 4 * (2 * w + i) + (lane >> 4), slot = lane & 15;
            const uint32_t rowoff = (uint32_t)(min(t0 + row, kend - 1) * kv_ss);
            const __bf16 *gk = kbase + rowoff + ((slot ^ (row & 15)) << 3);
            const __bf16 *gv = vbase + rowoff + ((slot ^ ((row & 3) << 2)) << 3);
            const uint32_t ldsk = lds0 + i * 1024, ldsv = ldsk + kKT * D * 2;
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(ldsk), "v"(gk) : "memory", "m0");
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(ldsv), "v"(gv) : "memory", "m0");
        }
    }
}

template <int D>
__global__ __launch_bounds__(kGsThreads) void tree_attn_ld_kernel(AttnArgs a) {
    constexpr int DB = D / 32;
    constexpr int TILE = 2 * kKT * D * 2;   // one K tile ([64][D] bf16, swizzled) + one V tile (row-major, swizzled)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int *s_par = reinterpret_cast<int *>(smem + kLdBufs * TILE);

    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int sp = blockIdx.x;
    // The blocks of units that share a range of cache rows are ranges x KV heads apart in workgroup number:
    // a multiple of eight with eight KV heads, and consecutive numbers go to consecutive XCDs, so the
    // blocks meet in one XCD's L2 and their rows come from HBM once.
    const int hk = blockIdx.y, ublk = blockIdx.z % a.n_ublk;
    const int b = blockIdx.z / a.n_ublk;
    const int L = a.ctx_lens[b];
    int nn = a.n_nodes ? a.n_nodes[b] : a.T;
    nn = max(1, min(nn, a.T));
    const int total = min(L + nn, a.S);                  // never read past the cache the caller described
    const int kbeg = sp * a.kps;
    if (L < 0 || kbeg >= total) return;
    const int kend = min(total, kbeg + a.kps);
    const int nsplit = (total + a.kps - 1) / a.kps;

    const int u = ublk * kGsWaves + w;                    // (head within the group, block of 32 rows)
    const int g = u / a.nqb, qb = u % a.nqb;
    const bool active = g < a.G;
    const int h = hk * a.G + (active ? g : 0);
    const int j32 = lane & 31, g2 = lane >> 5;
    const int i = 32 * qb + j32;                          // this lane's tree row

    const __bf16 *kbase = a.k + (size_t)b * a.kv_sb + (size_t)hk * a.kv_sh;
    const __bf16 *vbase = a.v + (size_t)b * a.kv_sb + (size_t)hk * a.kv_sh;
    const int kv_ss = (int)a.kv_ss;          // 32-bit offsets inside one head's cache (checked on the host)
    const int ntiles = (kend - kbeg + kKT - 1) / kKT;

    // the first two tiles are requested before anything else: the query rows below are consumed as soon as
    // they arrive, and loads issued behind that wait would start a memory round trip late
    const LdLane ldo = ld_lane_offsets<D>(kv_ss, w, lane);
    ld_issue_tile<D>(smem, kbase, vbase, kv_ss, kbeg, kend, w, lane, ldo);
    ld_issue_tile<D>(smem + TILE, kbase, vbase, kv_ss, kbeg + kKT, kend, w, lane, ldo);
    if (tid < RADAR_T_MAX) s_par[tid] = a.parents[(size_t)b * a.T + min(tid, nn - 1)];
    bf16x8 qop[D / 16];                                  // row i, d = 16*st + 8*g2 .. +8, for the whole kernel
    {
        const __bf16 *qrow = a.q + (size_t)b * a.q_sb + (size_t)h * a.q_sh + (uint32_t)(min(i, a.T - 1) * (int)a.q_st);
#pragma unroll
        for (int st = 0; st < D / 16; ++st) {
            u32x4 raw = *reinterpret_cast<const u32x4 *>(qrow + 16 * st + 8 * g2);
            and_mask(raw, active && i < a.T);
            qop[st] = __builtin_bit_cast(bf16x8, raw);
        }
    }
    __syncthreads();                                     // the parents are in LDS
    uint64_t anc[1];
    anc[0] = (kend > L && i < nn) ? ancestor_word(s_par, i) : 0ull;

    floatx16 oacc[DB][1];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][0][r] = 0.f;
    float m_run[1] = {kNegBig}, l_run[1] = {0.f};

    // Tiles are taken in pairs, four buffers: while the pair (t, t+1) is consumed from two of them the
    // loads of the next pair arrive in the other two.  One barrier per pair: it publishes the pair
    // (every wavefront has waited for its own loads) and tells that nobody reads the previous pair
    // any more, whose buffers the loads issued right after it overwrite -- issued whether or not the
    // range still has such tiles (see above).  (Not __syncthreads(): nothing here needs its fence.)
    // The two wavefronts of a SIMD (w and w + 4) are favoured in turn, one in the first tile of a pair
    // and the other in the second.  Left alone, the older wavefront wins the arbitration in every
    // tile and finishes it a third ahead of the other; taking turns measured 3-4 % faster at 16 K
    // cached rows.  (A barrier per pair without the priorities is slower than one per tile, and
    // priorities with a barrier per tile change nothing.)
    // Operand addresses: a lane's are the same in every tile up to the tile's place in LDS, so they are
    // kept in registers (eight for K: the XOR swizzle is not additive in the chunk; four for V) and the
    // sub-tile, the step inside the tile and the second tile of a pair are instruction offsets; only the
    // pair's own 64 KB step is added, once per pair.  (Recomputed per tile, as the compiler does when
    // handed a tile pointer, they were a quarter of the loop's vector instructions.)
    const lds_byte *ka[D / 16], *va[DB];
    {
        const lds_byte *base = (const lds_byte *)smem;
#pragma unroll
        for (int st = 0; st < D / 16; ++st) ka[st] = base + ks_off<D>(j32, 2 * st + g2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int d0 = 32 * db + (j32 & 16) + 4 * (lane & 3), kv0 = 4 * g2 + ((lane >> 2) & 3);
            va[db] = base + TILE / 2 + vs_off<D>(kv0, d0 >> 3) + (d0 & 7) * 2;
        }
    }
    floatx16 sacc[2];
    bf16x8 pk[2][2];
    auto run_tile = [&](auto second, int t0, bool first) {
        constexpr int TOFF = decltype(second)::value ? TILE : 0;
        // sub-tile k % 2: 32 rows on, the same swizzle (32 is a multiple of 16)
        tile_scores<D>([&](int k) { return (lds_u32x4)(ka[k >> 1] + TOFF + (k & 1) * (32 * D * 2)); }, qop, sacc);
        tile_softmax<D>(sacc, oacc, m_run[0], l_run[0], anc[0], t0, L, kend, first, a.scale_log2, pk);
        // step k: output block k % DB, rows 16 * (k / DB) on (a multiple of 4: the same swizzle), hi: 8 rows on
        tile_pv<D, true>([&](int k, int hi) { return va[k % DB] + TOFF + (k / DB) * (16 * D * 2) + hi * (8 * D * 2); }, pk, oacc);
    };
    const int fav = w < kGsWaves / 2 ? 1 : 0;
    for (int t = 0; t < ntiles; t += 2) {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const int half = (t >> 1) & 1;                                     // this pair sits in buffers 2*half, 2*half + 1
        ld_issue_tile<D>(smem + (2 - 2 * half) * TILE, kbase, vbase, kv_ss, kbeg + (t + 2) * kKT, kend, w, lane, ldo);
        ld_issue_tile<D>(smem + (3 - 2 * half) * TILE, kbase, vbase, kv_ss, kbeg + (t + 3) * kKT, kend, w, lane, ldo);
        if (active) {
            if (fav) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
            run_tile(std::false_type{}, kbeg + t * kKT, t == 0);
            if (fav) __builtin_amdgcn_s_setprio(0); else __builtin_amdgcn_s_setprio(1);
            if (t + 1 < ntiles) run_tile(std::true_type{}, kbeg + (t + 1) * kKT, false);
        }
        const int step = half ? -2 * TILE : 2 * TILE;                     // the next pair sits in the other two buffers
#pragma unroll
        for (int st = 0; st < D / 16; ++st) ka[st] += step;
#pragma unroll
        for (int db = 0; db < DB; ++db) va[db] += step;
    }
    __builtin_amdgcn_s_setprio(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // nothing may still be on its way into LDS at the end
    if (!active) return;
    gs_finish<D>(a, [&](int db, int r) { return oacc[db][0][r]; }, m_run[0], l_run[0], b, h, i, nn, sp, nsplit);
}

// Merges the group-share kernel's per-split partials.  A workgroup takes one (sequence, query
// head, 32-wide slice of the head dimension): lane = (tree row i, 8 consecutive d), so that the
// reads of a d-row of the [D][64] partial are 256 contiguous bytes.  Splits are taken four at a
// time so that a batch's loads are in flight together.
template <int D>
__global__ __launch_bounds__(kAttnThreads) void tree_attn_merge_kernel(AttnArgs a) {
    constexpr int SL = 32, DQ = 8;                          // slice width, floats per lane
    const int slice = blockIdx.x % (D / SL), h = blockIdx.x / (D / SL), b = blockIdx.y;
    const int L = a.ctx_lens[b];
    int nn = a.n_nodes ? a.n_nodes[b] : a.T;
    nn = max(1, min(nn, a.T));
    const int total = min(L + nn, a.S);
    const int nsplit = (total + a.kps - 1) / a.kps;
    if (L < 0 || nsplit <= 1) return;                       // the split kernel wrote the result itself

    const int i = threadIdx.x & 63, part = threadIdx.x >> 6; // query row, which 8 of the slice's 32
    if (i >= a.T) return;
    const int d0 = slice * SL + part * DQ;
    const size_t unit0 = ((size_t)b * a.Hq + h) * a.max_splits;
    __bf16 *orow = a.out + (size_t)b * a.o_sb + (size_t)i * a.o_st + (size_t)h * a.o_sh + d0;
    const bool lse_lane = a.lse && slice == 0 && part == 0;
    if (i >= nn) {
        bf16x8 z;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = (__bf16)0.f;
        *reinterpret_cast<bf16x8 *>(orow) = z;
        if (lse_lane) a.lse[((size_t)b * a.T + i) * a.Hq + h] = 0.f;
        return;
    }
    float M = kNegBig, lsum = 0.f;
    float acc[DQ];
#pragma unroll
    for (int d = 0; d < DQ; ++d) acc[d] = 0.f;
    for (int s0 = 0; s0 < nsplit; s0 += 4) {
        float ms[4], ls[4];
        uint32_t ow[4][DQ / 2];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int sc = min(s0 + j, nsplit - 1);
            ms[j] = a.part_ml[(unit0 + sc) * 192 + i];
            ls[j] = a.part_ml[(unit0 + sc) * 192 + 64 + i] * a.part_ml[(unit0 + sc) * 192 + 128 + i];   // l x magnitude
            const uint32_t *po = a.part_o + (unit0 + sc) * (size_t)(D / 2 * 64);
#pragma unroll
            for (int d = 0; d < DQ / 2; ++d) ow[j][d] = po[((d0 >> 1) + d) * 64 + i];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool valid = s0 + j < nsplit;
            const float m = valid ? ms[j] : kNegBig;
            const float Mn = fmaxf(M, m);
            const float aold = __builtin_amdgcn_exp2f(M - Mn);
            const float wnew = valid ? __builtin_amdgcn_exp2f(m - Mn) : 0.f;
            const float lj = a.part_ml[(unit0 + min(s0 + j, nsplit - 1)) * 192 + 64 + i];
            lsum = lsum * aold + wnew * lj;
            const float wo = wnew * ls[j];                        // the stored rows are o / (l x magnitude)
#pragma unroll
            for (int d = 0; d < DQ / 2; ++d) {
                const float lo = (float)__builtin_bit_cast(_Float16, (uint16_t)(ow[j][d] & 0xffffu));
                const float hi = (float)__builtin_bit_cast(_Float16, (uint16_t)(ow[j][d] >> 16));
                acc[2 * d] = acc[2 * d] * aold + wo * lo;
                acc[2 * d + 1] = acc[2 * d + 1] * aold + wo * hi;
            }
            M = Mn;
        }
    }
    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
    bf16x8 o8;
#pragma unroll
    for (int e = 0; e < 8; ++e) o8[e] = (__bf16)(acc[e] * inv);
    *reinterpret_cast<bf16x8 *>(orow) = o8;
    if (lse_lane) a.lse[((size_t)b * a.T + i) * a.Hq + h] = (M + __builtin_amdgcn_logf(lsum)) * kLn2;
}

// ------------------------------------------------------------------ host-side planning
struct AttnPlan {
    int kps, max_splits, n_ublk, nqb;
    size_t off_part_o, off_part_ml, bytes;
};

static AttnPlan plan_attention(const radar_attn_desc *d) {
    AttnPlan p;
    const int G = d->Hq / d->Hkv;
    p.nqb = d->T_max <= 32 ? 1 : 2;
    p.n_ublk = (G * p.nqb + kGsWaves - 1) / kGsWaves;
    long kps = d->keys_per_split;
    if (kps <= 0) {
        // Number of key ranges: the one that minimises a small cost model, in units of one tile of
        // one workgroup (measured ~2.7 us): rounds of 256 resident workgroups x (tiles per range +
        // 3 for prologue and epilogue), plus what the merge of the ranges costs (every range writes
        // and re-reads T*Hq*D fp16 of partial output, which soon exceeds the KV bytes themselves).
        // Counting whole rounds matters: 576 workgroups take as long as 768.
        const long units = (long)d->B * d->Hkv * p.n_ublk;
        const long tiles_all = ((long)d->S_max + kKT - 1) / kKT;
        double best = 1e30;
        long best_ns = 1;
        for (long ns = 1; ns <= 64 && ns <= tiles_all; ++ns) {
            const long tiles = (tiles_all + ns - 1) / ns;
            const long rounds = (units * ns + 255) / 256;
            const double cost = (double)rounds * (double)(tiles + 3) + (ns > 1 ? 1.6 + 0.3 * (double)ns : 0.0);
            if (cost < best) { best = cost; best_ns = ns; }
        }
        kps = (tiles_all + best_ns - 1) / best_ns * kKT;
    }
    p.kps = (int)kps;
    p.max_splits = (int)(((long)d->S_max + kps - 1) / kps);
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += (bytes + 255) & ~size_t(255); return o; };
    take(256);                                             // never empty: callers always pass a workspace
    const size_t units = p.max_splits > 1 ? (size_t)d->B * d->Hq * p.max_splits : 0;
    p.off_part_o = take(units * 64 * (d->D / 2) * sizeof(uint32_t));
    p.off_part_ml = take(units * 192 * sizeof(float));
    p.bytes = off;
    return p;
}

}  // namespace radar

using namespace radar;

static radar_status check_attn_desc(const radar_attn_desc *d) {
    if (!d) return RADAR_INVALID_ARG;
    if (d->B < 1 || d->T_max < 1 || d->Hq < 1 || d->Hkv < 1 || d->S_max < 1 || d->Hq % d->Hkv != 0)
        return RADAR_INVALID_ARG;
    if (d->keys_per_split < 0 || d->keys_per_split % kKT != 0) return RADAR_INVALID_ARG;
    if (d->softmax_scale < 0.f) return RADAR_INVALID_ARG;
    if ((d->D != 64 && d->D != 128) || d->T_max > RADAR_T_MAX) return RADAR_UNSUPPORTED_SHAPE;
    if (d->B > 65535 || d->Hq > 65535) return RADAR_UNSUPPORTED_SHAPE;
    return RADAR_OK;
}

extern "C" size_t radar_tree_attention_workspace_bytes(const radar_attn_desc *d) {
    if (check_attn_desc(d) != RADAR_OK) return 0;
    return plan_attention(d).bytes;
}

template <int D>
constexpr int gs_smem_bytes() { return 2 * (2 * kKT * D * 2) + RADAR_T_MAX * 4; }

template <int D>
static hipError_t launch_ld(const AttnArgs &a, dim3 grid, hipStream_t s) {
    constexpr int bytes = kLdBufs * (2 * kKT * D * 2) + RADAR_T_MAX * 4;
    static const hipError_t configured = hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_attn_ld_kernel<D>),
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (configured != hipSuccess) return configured;
    return launch("tree_attn_group_share", tree_attn_ld_kernel<D>, grid, dim3(kGsThreads), bytes, s, a);
}

template <int D, bool DEEP>
static hipError_t launch_gs(const AttnArgs &a, dim3 grid, hipStream_t s) {
    // the dynamic LDS limit is raised once per instantiation (a function-local static is initialised
    // exactly once, also when several threads launch at the same time)
    static const hipError_t configured = hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_attn_gs_kernel<D, DEEP>),
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, gs_smem_bytes<D>());
    if (configured != hipSuccess) return configured;
    return launch("tree_attn_group_share", tree_attn_gs_kernel<D, DEEP>, grid, dim3(kGsThreads), gs_smem_bytes<D>(), s, a);
}

extern "C" radar_status radar_tree_attention(const void *q, const void *k_cache, const void *v_cache,
                                             const int32_t *parents, const int32_t *ctx_lens, const int32_t *n_nodes,
                                             void *out, float *lse_out, const radar_attn_desc *d, void *workspace,
                                             size_t workspace_bytes, void *stream) {
    if (!q || !k_cache || !v_cache || !parents || !ctx_lens || !out || !workspace) return RADAR_INVALID_ARG;
    radar_status st = check_attn_desc(d);
    if (st != RADAR_OK) return st;
    const AttnPlan p = plan_attention(d);
    if (workspace_bytes < p.bytes) return RADAR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return RADAR_INVALID_ARG;

    AttnArgs a;
    a.q = static_cast<const __bf16 *>(q); a.k = static_cast<const __bf16 *>(k_cache);
    a.v = static_cast<const __bf16 *>(v_cache);
    a.parents = parents; a.ctx_lens = ctx_lens; a.n_nodes = n_nodes;
    a.out = static_cast<__bf16 *>(out); a.lse = lse_out;
    a.B = d->B; a.T = d->T_max; a.Hq = d->Hq; a.Hkv = d->Hkv; a.G = d->Hq / d->Hkv; a.S = d->S_max;
    a.kps = p.kps; a.max_splits = p.max_splits; a.n_ublk = p.n_ublk; a.nqb = p.nqb;
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
    // the kernels address rows inside one head's cache / one head's queries with 32-bit offsets
    if (a.kv_ss <= 0 || a.q_st <= 0 || a.kv_ss * (int64_t)d->S_max >= (int64_t(1) << 31) ||
        a.q_st * (int64_t)d->T_max >= (int64_t(1) << 31))
        return RADAR_UNSUPPORTED_SHAPE;
    const float scale = d->softmax_scale != 0.f ? d->softmax_scale : 1.0f / sqrtf((float)d->D);
    a.scale_log2 = scale * kLog2e;
    char *ws = static_cast<char *>(workspace);
    a.part_o = reinterpret_cast<uint32_t *>(ws + p.off_part_o);
    a.part_ml = reinterpret_cast<float *>(ws + p.off_part_ml);

    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 block(kAttnThreads);
    if ((long)a.B * a.n_ublk > 65535) return RADAR_UNSUPPORTED_SHAPE;
    const dim3 grid((unsigned)a.max_splits, (unsigned)a.Hkv, (unsigned)(a.B * a.n_ublk));
    {
        hipError_t e;
        if (p.kps >= 8 * kKT) e = d->D == 128 ? launch_ld<128>(a, grid, s) : launch_gs<64, true>(a, grid, s);
        else                  e = d->D == 128 ? launch_gs<128, false>(a, grid, s) : launch_gs<64, false>(a, grid, s);
        if (e != hipSuccess) return RADAR_HIP_ERROR;
    }
    if (a.max_splits > 1) {
        const dim3 mgrid((unsigned)(a.Hq * (d->D / 32)), (unsigned)a.B);
        const hipError_t e = d->D == 128 ? launch("tree_attn_merge", tree_attn_merge_kernel<128>, mgrid, block, 0, s, a)
                                         : launch("tree_attn_merge", tree_attn_merge_kernel<64>, mgrid, block, 0, s, a);
        if (e != hipSuccess) return RADAR_HIP_ERROR;
    }
    return RADAR_OK;
}
