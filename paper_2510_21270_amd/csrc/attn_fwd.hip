// pbs_attn_fwd: Algorithm 1's main loop -- online-softmax attention over the listed key blocks only.
// This file holds the entry point, the 32-queries-per-wave matrix-core kernel and the vector kernel; the
// 64-queries-per-wave kernel that serves block = 128 first is in attn_wide.hip.
//
// Matrix-core kernel (bf16, d = 128; block 64, and the second pass of block 128).  Everything is kept TRANSPOSED so
// that one lane owns one query for the whole row of work:
//     S^T = K'_j Q'_i^T      A = K' tile rows (from LDS), B = Q' fragments (registers, loaded once)
//     O^T += V'_j^T P^T      A = V'^T tile rows (from LDS; V' is stored block-transposed in HBM), B = P^T
// With v_mfma_f32_32x32x16_bf16 the accumulator of S^T gives lane (n, h) the scores of query n against 16 keys
// of every 32-key tile, which after exp2 and a bf16 pack IS the B operand of the second product -- no
// cross-lane traffic for P, and the running max / sum / rescale of a query are lane-local (one xor-32
// exchange).  The K' tile is stored in LDS with bits 2 and 3 of the row index swapped so that the 8 values a
// lane contributes to one 16-key contraction step are 8 CONSECUTIVE keys, which lets V'^T be read from LDS
// with plain 16-byte loads.  LDS tile rows are padded by 16 bytes against bank conflicts.
// A block that is not listed costs nothing: the loop runs over the list.
//
// Vector kernel (fp32 arithmetic): every other supported dtype / d / block.
#include <limits.h>

#include "pbs_host.h"

namespace pbs {

constexpr float kLog2eF = 1.4426950408889634f;
constexpr float kLn2F = 0.6931471805599453f;

__device__ inline int swap23(int m) { return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1); }

// ---------------------------------------------------------------------------------------------
// MFMA kernel.  BLOCK = block size; WAVES = waves per workgroup; each wave owns BLOCK / WAVES query rows.
// Key blocks are consumed in sub-tiles of KT keys (64 for block 128; 32 for block 64, whose two-wave workgroups then
// need 39 KB of LDS, so that four of them -- two waves per SIMD -- share a CU).  K' and V'^T sub-tiles are double-buffered in LDS and
// filled by asynchronous buffer->LDS loads (no registers, no LDS store instructions): while sub-tile s is being
// multiplied, sub-tile s+1 is in flight.  One barrier per sub-tile.
// grid = 1-D, see the workgroup decoding at the top of the kernel.
//
// Softmax with a lazily updated reference.  On the common path an element costs one v_fma_f32 (s*c - mref), one
// v_exp_f32, and per pair one v_cvt_pk_bf16_f32 and one v_dot2c_f32_bf16 (row sum of the ROUNDED probabilities):
// no row maximum, no rescale of O.  Any reference gives the same softmax as long as nothing overflows, so the
// reference only has to move when a row sum grows past 2^16; that, a block that needs the token-level causal
// mask, and a query that has not met a visible key yet take the exact path (row maximum, reference update,
// rescale of O and l).
// ---------------------------------------------------------------------------------------------
constexpr int kListChunk = 256;                            // listed blocks staged in LDS at a time
constexpr int kXcds = 8;                                   // accelerator dies, each with a private L2
constexpr int kCohort = 64;                                // workgroups resident per XCD (32 CUs x 2)
constexpr float kBigRowSum = 65536.0f;                     // lazy-reference overflow guard

typedef __attribute__((address_space(3))) void *lptr_t;

// Buffer descriptors (base, size in bytes) of one kv head's K', V'^T and key positions.  A load is
// "descriptor base + scalar tile offset + per-lane offset": no 64-bit vector arithmetic, and anything past the end
// of K' or of the positions reads as zero (such key slots are rejected by index in the exact softmax path).
struct TileBuffers {
    __amdgpu_buffer_rsrc_t k, v, pos;
};

template <int BLOCK>
__device__ inline TileBuffers tile_buffers(const bf16_t *Kh, const bf16_t *Vh, const int32_t *kih, int n, int T)
{
    constexpr int kRawDword = 0x00020000;                  // gfx9 descriptor word 3: raw 32-bit data format
    TileBuffers b;
    b.k = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(Kh), 0, n * 256, kRawDword);
    b.v = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(Vh), 0, T * 128 * BLOCK * 2, kRawDword);
    b.pos = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(kih), 0, n * 4, kRawDword);
    return b;
}

// LDS tiles are row-padded by 16 bytes instead of XOR-swizzled: K' sub-tile rows are 272 bytes (256 + 16), V'^T
// sub-tile rows 144 bytes (128 + 16).  Sixteen consecutive rows then start 4 (resp. 36 mod 64) banks apart, so the
// 16-lane groups of a ds_read_b128 hit 64 distinct banks, and -- unlike a swizzle -- the address of fragment k is
// "lane base + k * 32 bytes", an immediate offset: one address register per tile instead of one per fragment.
// LDS row r of the K' tile holds key (r & ~31) | swap23(r & 31).
constexpr int kKRowB = 272;                                // padded K' row in bytes
template <int KT>
struct SubTile {
    static constexpr int kVRowB = KT * 2 + 16;             // padded V'^T row: 144 (KT = 64) or 80 bytes (KT = 32)
    static constexpr int kKLoads = (KT * kKRowB + 1023) / 1024;   // 1 KiB load chunks: 17 or 9 (the last half used)
    static constexpr int kVLoads = 128 * kVRowB / 1024;    // 18 or 10
    static constexpr int kKTileB = kKLoads * 1024, kVTileB = kVLoads * 1024;
};

// Per-lane global byte offsets of this wave's chunks inside a sub-tile, computed once.  One load instruction
// moves 64 lanes x 16 bytes into 1 KiB of CONTIGUOUS LDS; the lane decides which global chunk lands there, so the
// LDS image is the padded tile (lanes that fall on padding bytes fetch chunk 0 of their row, harmlessly).
template <int WAVES, int KT>
struct LaneOffsets {
    uint32_t k[(SubTile<KT>::kKLoads + WAVES - 1) / WAVES], v[(SubTile<KT>::kVLoads + WAVES - 1) / WAVES];
};

template <int BLOCK, int WAVES, int KT>
__device__ inline LaneOffsets<WAVES, KT> lane_offsets(int wave, int lane)
{
    typedef SubTile<KT> ST;
    LaneOffsets<WAVES, KT> o;
#pragma unroll
    for (int y = 0; y < (ST::kKLoads + WAVES - 1) / WAVES; ++y) {
        const int pos = (wave + WAVES * y) * 1024 + lane * 16;
        const int r = pos / kKRowB, col = pos % kKRowB;
        const int key = (r & ~31) | swap23(r & 31);
        o.k[y] = r < KT ? (uint32_t)(key * 256 + (col < 256 ? col : 0)) : 0u;   // past the tile: padding of the chunk
    }
#pragma unroll
    for (int y = 0; y < (ST::kVLoads + WAVES - 1) / WAVES; ++y) {
        const int pos = (wave + WAVES * y) * 1024 + lane * 16;
        const int r = pos / ST::kVRowB, col = pos % ST::kVRowB;
        // Vt: groups of 32 keys, each [128 features][32 keys]; a sub-tile is KT / 32 consecutive groups
        o.v[y] = (uint32_t)(col < KT * 2 ? ((col >> 6) * 128 + r) * 64 + (col & 63) : r * 64);
    }
    return o;
}

// Index remapping (appendix "Memory Overhead": the kernel retrieves the keys directly from the original tensor through
// the permuted indices): the rows of a K' sub-tile are rows kidx[slot] of the caller's K.  A lane needs the index of
// the one row it moves in each of its load chunks; KeyRows holds them for one sub-tile, fetched one sub-tile ahead of
// the loads that use them (they arrive under the multiplication of the sub-tile in between).
template <int WAVES, int KT>
struct KeyRows {
    int row[(SubTile<KT>::kKLoads + WAVES - 1) / WAVES];
};

// kidx entries of the rows this lane moves for the sub-tile at `half` of block j (slots past n read as 0: row 0,
// whose scores are discarded by the slot test like those of any slot past n)
template <int BLOCK, int WAVES, int KT>
__device__ inline void fetch_key_rows(KeyRows<WAVES, KT> &kr, const TileBuffers &buf, const LaneOffsets<WAVES, KT> &off,
                                      int j, int half)
{
    const int slot0 = j * BLOCK + half * KT;
#pragma unroll
    for (int y = 0; y < (SubTile<KT>::kKLoads + WAVES - 1) / WAVES; ++y)
        kr.row[y] = __builtin_amdgcn_raw_buffer_load_b32(buf.pos, (off.k[y] >> 8) * 4, slot0 * 4, 0);
}

template <int BLOCK, int WAVES, int KT, bool REMAP>
__device__ inline void issue_subtile(unsigned char *kbuf, unsigned char *vbuf, int *kpos, const TileBuffers &buf,
                                     const LaneOffsets<WAVES, KT> &off, const KeyRows<WAVES, KT> &kr, int j, int half,
                                     bool masked, int wave, int lane)
{
    constexpr int kKLoads = SubTile<KT>::kKLoads, kVLoads = SubTile<KT>::kVLoads;
    const int slot0 = j * BLOCK + half * KT;               // uniform
    // full rounds are unconditional; only the last, partial round of chunks tests the wave index
#pragma unroll
    for (int y = 0; y < (kKLoads + WAVES - 1) / WAVES; ++y)
        if (y < kKLoads / WAVES || wave < kKLoads % WAVES) {
            if (REMAP)                                     // buf.k is the caller's K: row kidx[slot], same 16-byte piece
                __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.k, (lptr_t)(kbuf + (wave + WAVES * y) * 1024), 16,
                                                         (uint32_t)kr.row[y] * 256u + (off.k[y] & 255u), 0, 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.k, (lptr_t)(kbuf + (wave + WAVES * y) * 1024), 16, off.k[y],
                                                         slot0 * 256, 0, 0);
        }
#pragma unroll
    for (int y = 0; y < (kVLoads + WAVES - 1) / WAVES; ++y)
        if (y < kVLoads / WAVES || wave < kVLoads % WAVES)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.v, (lptr_t)(vbuf + (wave + WAVES * y) * 1024), 16, off.v[y],
                                                     j * (128 * BLOCK * 2) + half * (128 * KT * 2), 0, 0);
    if (masked && wave == WAVES - 1)                       // original positions of 64 keys from the sub-tile's first on
        __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.pos, (lptr_t)kpos, 4, lane * 4, slot0 * 4, 0, 0);
}

// Barrier that also publishes the asynchronous LDS loads of every wave: the loads of a wave are only counted by
// that wave's own vmcnt, and the workgroup-scope fence of __syncthreads() does not wait on them, so each wave
// drains its own counter (s_waitcnt vmcnt(0), gfx9 encoding) before it arrives at the barrier.
__device__ inline void sync_tiles()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
}

template <int NT>
struct AttnState {
    floatx16 acc_o[4][NT];
    float mref[NT], l[NT];  // reference (log2 units) and sum of exp2(s*c - mref), this lane's half of the keys
    bool seen[NT];          // the query has met at least one visible key, i.e. mref is meaningful
};

// p = exp2(s * c2 - shift) for 8 consecutive keys, packed to bf16.  PLAIN_SUM = false: rsum += the rounded values,
// one bf16 dot-product instruction per pair; true: rsum += the unrounded values, two additions per pair, which
// overlap better with matrix instructions but need two more registers (the four-wave instantiation has none to spare).
template <bool PLAIN_SUM>
__device__ inline bf16x8 exp2_pack8(const floatx16 &s, int base, float c2, float shift, float &rsum)
{
    const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
    bf16x8 pk;
    float odd = 0.0f;
#pragma unroll
    for (int y = 0; y < 4; ++y) {
        floatx2 pr = {__builtin_amdgcn_exp2f(__builtin_fmaf(s[base + 2 * y], c2, -shift)),
                      __builtin_amdgcn_exp2f(__builtin_fmaf(s[base + 2 * y + 1], c2, -shift))};
        const bf16x2 t2 = __builtin_convertvector(pr, bf16x2);
        if (PLAIN_SUM) {
            rsum += pr[0];
            odd += pr[1];
        } else {
            rsum = __builtin_amdgcn_fdot2_f32_bf16(t2, ones, rsum, false);
        }
        pk[2 * y] = t2[0];
        pk[2 * y + 1] = t2[1];
    }
    if (PLAIN_SUM) rsum += odd;
    return pk;
}

// One sub-tile: S^T = K' Q'^T, softmax relative to the lane's reference, O^T += V'^T P^T.
template <int BLOCK, int NT, int KT>
__device__ inline void compute_subtile(AttnState<NT> &st, const unsigned char *kbuf, const unsigned char *vbuf,
                                       const bf16x8 (&qf)[NT][8], const int (&qpos)[NT], const int *kpos, int room,
                                       bool masked, float c2, int ln, int lh)
{
    constexpr int MT = KT / 32;                                  // 32-key tiles per sub-tile
    constexpr int KS = KT / 16;                                  // 16-key contraction steps per sub-tile
    constexpr int kVRowB = SubTile<KT>::kVRowB;
    const unsigned char *kl = kbuf + ln * kKRowB + lh * 16;      // this lane's row / half inside a 32-key tile
    const unsigned char *vl = vbuf + ln * kVRowB + lh * 16;
    // S^T of one 32-key tile (8 MFMAs per query tile).  Operand fragments are fetched from LDS four at a time
    // (16 registers), the next four while the current four are being multiplied; the scheduling barriers keep the
    // compiler from hoisting every load to the top (registers) or sinking each one next to its MFMA (latency).
    auto s_tile = [&](floatx16 (&acc)[NT], int mt) {
        bf16x8 fa[4], fb[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) fa[x] = *reinterpret_cast<const bf16x8 *>(kl + mt * 32 * kKRowB + x * 32);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int x = 0; x < 4; ++x) fb[x] = *reinterpret_cast<const bf16x8 *>(kl + mt * 32 * kKRowB + (4 + x) * 32);
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[x], qf[nt][x], x == 0 ? floatx16{0} : acc[nt], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[x], qf[nt][4 + x], acc[nt], 0, 0, 0);
    };
    // acc[nt][x] of tile mt: key (within the sub-tile) = 32 mt + 16 (x / 8) + 8 h + (x % 8), query = q0 + 32 nt + n

    bf16x8 pf[NT][KS];
    bool all_seen = true;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) all_seen = all_seen && st.seen[nt];
    bool exact = masked || !__all(all_seen);
    if (!exact) {
        // common path: p = exp2(S), one 32-key tile at a time (the scores of a tile die as soon as they are packed)
        float rsum[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) rsum[nt] = 0.0f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            floatx16 acc[NT];
            s_tile(acc, mt);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int u = 0; u < 2; ++u) pf[nt][2 * mt + u] = exp2_pack8<KT == 32>(acc[nt], 8 * u, c2, st.mref[nt], rsum[nt]);
        }
        bool big = false;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) big = big || !(rsum[nt] <= kBigRowSum);
        if (__any(big)) {
            exact = true;                                  // a row outgrew its reference: redo this sub-tile exactly
        } else {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) st.l[nt] += rsum[nt];
        }
    }
    if (exact) {
        floatx16 acc_s[MT][NT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) s_tile(acc_s[mt], mt);
        if (masked) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int k8 = 32 * mt + 16 * u + 8 * lh;  // 8 consecutive keys of this lane
                    const int4 a = *reinterpret_cast<const int4 *>(kpos + k8);
                    const int4 b = *reinterpret_cast<const int4 *>(kpos + k8 + 4);
                    const int kp[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                    const int lim = room - k8;                 // keys x >= lim of this group do not exist
#pragma unroll
                    for (int x = 0; x < 8; ++x)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            if (kp[x] > qpos[nt] || x >= lim) acc_s[mt][nt][8 * u + x] = -INFINITY;
                }
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float rmax = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int x = 0; x < 16; ++x) rmax = fmaxf(rmax, acc_s[mt][nt][x]);
            rmax = fmaxf(rmax, __shfl_xor(rmax, 32, 64));
            const bool was = st.seen[nt];
            const bool now = was || rmax != -INFINITY;
            // move the reference up to the row maximum (first contact: set it to the maximum, whatever its sign)
            const float mnew = now ? (was ? fmaxf(rmax * c2, st.mref[nt]) : rmax * c2) : 0.0f;
            const float alpha = was ? __builtin_amdgcn_exp2f(st.mref[nt] - mnew) : 1.0f;
            float rsum = 0.0f;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int u = 0; u < 2; ++u) pf[nt][2 * mt + u] = exp2_pack8<KT == 32>(acc_s[mt][nt], 8 * u, c2, mnew, rsum);
            st.l[nt] = st.l[nt] * alpha + rsum;
            st.seen[nt] = now;
            st.mref[nt] = mnew;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int x = 0; x < 16; ++x) st.acc_o[dt][nt][x] *= alpha;
            }
        }
    }

    {
        bf16x8 fa[KS], fb[KS];
#pragma unroll
        for (int x = 0; x < KS; ++x) fa[x] = *reinterpret_cast<const bf16x8 *>(vl + x * 32);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {                   // one 32-row tile of O^T per step, KS fragments each
            bf16x8(&cur)[KS] = (dt & 1) ? fb : fa;
            bf16x8(&nxt)[KS] = (dt & 1) ? fa : fb;
            __builtin_amdgcn_sched_barrier(0);
            if (dt < 3) {
#pragma unroll
                for (int x = 0; x < KS; ++x)
                    nxt[x] = *reinterpret_cast<const bf16x8 *>(vl + (dt + 1) * 32 * kVRowB + x * 32);
            }
#pragma unroll
            for (int k2 = 0; k2 < KS; ++k2)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    st.acc_o[dt][nt] =
                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur[k2], pf[nt][k2], st.acc_o[dt][nt], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// REMAP: Kp is the caller's K in token order and the K' sub-tiles are gathered from it through kidx (index remapping).
template <int BLOCK, int WAVES, int KT, bool REMAP = false>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_mfma_kernel(
    const bf16_t *__restrict__ Qp, const bf16_t *__restrict__ Kp, const bf16_t *__restrict__ Vt,
    const int32_t *__restrict__ qidx, const int32_t *__restrict__ kidx, const int32_t *__restrict__ row_cnt,
    const int32_t *__restrict__ col_idx, bf16_t *__restrict__ Op, float *__restrict__ lse,
    const int32_t *__restrict__ only, Geo g)
{
    constexpr int D = 128;
    constexpr int NT = BLOCK / WAVES / 32;         // 32-query tiles per wave
    constexpr int SUBS = BLOCK / KT;               // sub-tiles per key block
    static_assert(NT >= 1 && SUBS >= 1, "unsupported tiling");

    __shared__ __align__(16) unsigned char kbuf0[SubTile<KT>::kKTileB], kbuf1[SubTile<KT>::kKTileB];   // 17 / 9 KiB each
    __shared__ __align__(16) unsigned char vbuf0[SubTile<KT>::kVTileB], vbuf1[SubTile<KT>::kVTileB];   // 18 / 10 KiB each
    __shared__ __align__(16) int kpos0[64], kpos1[64];
    __shared__ int jl[kListChunk];                                            // validated block list, -1 = skip

    // Workgroup -> (query head, query block).  Workgroups are handed to the 8 XCDs round-robin by linear id and
    // every XCD has its own L2, so the id is decoded as (xcd, slot): the 64 workgroups that are resident on one XCD
    // at a time form a cohort of 64 rows of ONE kv head with nearly equal list lengths (16 consecutive query blocks
    // x the r query heads of the group, longest first).  A cohort walks its ascending lists in near lock-step, so a
    // K'/V' sub-tile is fetched into that L2 once and hit by the other members.
    const int nbk = g.batch * g.h_kv;
    const int rows_per_unit = g.r * g.T;
    const int coh_per_unit = (rows_per_unit + kCohort - 1) / kCohort;
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int coh = (slot / kCohort) * kXcds + xcd;
    if (coh >= nbk * coh_per_unit) return;
    const int unit = coh % nbk;
    const int mrow = (coh / nbk) * kCohort + slot % kCohort;
    if (mrow >= rows_per_unit) return;
    const int i = g.T - 1 - mrow / g.r;
    const int b = unit / g.h_kv, hq = (unit % g.h_kv) * g.r + mrow % g.r;
    const int bhq = b * g.h_q + hq;
    if (only && only[(size_t)bhq * g.T + i] == 0) return;    // second pass: only the query blocks flagged by the first
    const size_t bhk = unit;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ln = lane & 31, lh = lane >> 5;
    const int q0 = i * BLOCK + wave * (BLOCK / WAVES);
    const float c2 = g.scale * kLog2eF;

    // Q' fragments: lane (n, h) holds Q'[q0 + 32 nt + n][16 ks + 8 h .. +8]
    bf16x8 qf[NT][8];
    int qpos[NT];
    AttnState<NT> st;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int qs = q0 + 32 * nt + ln;
        const int qc = qs < g.n ? qs : g.n - 1;
        const bf16_t *src = Qp + ((size_t)bhq * g.n + qc) * D + 8 * lh;
#pragma unroll
        for (int k = 0; k < 8; ++k) qf[nt][k] = *reinterpret_cast<const bf16x8 *>(src + 16 * k);
        qpos[nt] = qs < g.n ? (qidx ? qidx[(size_t)bhq * g.n + qs] : qs) : -1;
        st.mref[nt] = 0.0f;
        st.l[nt] = 0.0f;
        st.seen[nt] = qs >= g.n;                  // padding rows never hold the wave on the exact path
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int x = 0; x < 16; ++x) st.acc_o[dt][nt][x] = 0.0f;
    }

    const int ni = allowed_cols(i, g);
    const int jmask = first_masked_col(i, g);
    const int cnt = min(row_cnt[(size_t)bhq * g.T + i], g.T);
    const int32_t *cols = col_idx + ((size_t)bhq * g.T + i) * g.T;
    const TileBuffers buf = tile_buffers<BLOCK>(Kp + bhk * (size_t)g.n * D, Vt + bhk * (size_t)g.T * D * BLOCK,
                                                kidx + bhk * (size_t)g.n, g.n, g.T);
    const LaneOffsets<WAVES, KT> off = lane_offsets<BLOCK, WAVES, KT>(wave, lane);

    // The list is consumed in chunks staged in LDS (read back with LDS loads, which do not wait on the
    // asynchronous tile loads).  Entries outside the columns the causal mask admits become -1 and are skipped;
    // every test on them is uniform across the workgroup.  Sub-tile s of a chunk covers half (s % SUBS) of listed
    // block jl[s / SUBS].
    for (int base = 0; base < cnt; base += kListChunk) {
        const int len = min(kListChunk, cnt - base);
        __syncthreads();                   // previous chunk fully consumed
        for (int t = threadIdx.x; t < len; t += WAVES * 64) {
            const int j = cols[base + t];
            jl[t] = (j >= 0 && j < ni) ? j : -1;
        }
        __syncthreads();
        const int total = len * SUBS;
        auto block_at = [&](int s) -> int { return __builtin_amdgcn_readfirstlane(jl[s / SUBS]); };
        // with index remapping: the key rows of the sub-tile whose loads are issued next
        KeyRows<WAVES, KT> kr;
        auto fetch_rows = [&](int s) {
            if (REMAP && s < total) {
                const int js = block_at(s);
                if (js >= 0) fetch_key_rows<BLOCK, WAVES, KT>(kr, buf, off, js, s % SUBS);
            }
        };
        fetch_rows(0);
        {
            const int j0 = block_at(0);
            if (j0 >= 0)
                issue_subtile<BLOCK, WAVES, KT, REMAP>(kbuf0, vbuf0, kpos0, buf, off, kr, j0, 0, j0 >= jmask, wave, lane);
            fetch_rows(1);
        }
        for (int s = 0; s < total; s += 2) {
            sync_tiles();                  // sub-tile s has landed in buffer 0; buffer 1 is free again (and the key
                                           // rows of sub-tile s + 1 have arrived: the wait covers every load)
            if (s + 1 < total) {
                const int j1 = block_at(s + 1);
                if (j1 >= 0)
                    issue_subtile<BLOCK, WAVES, KT, REMAP>(kbuf1, vbuf1, kpos1, buf, off, kr, j1, (s + 1) % SUBS,
                                                           j1 >= jmask, wave, lane);
            }
            fetch_rows(s + 2);
            {
                const int j = block_at(s);
                if (j >= 0)
                    compute_subtile<BLOCK, NT, KT>(st, kbuf0, vbuf0, qf, qpos, kpos0, g.n - j * BLOCK - (s % SUBS) * KT,
                                               j >= jmask, c2, ln, lh);
            }
            if (s + 1 >= total) break;
            sync_tiles();                  // sub-tile s+1 has landed in buffer 1; buffer 0 is free again
            if (s + 2 < total) {
                const int j2 = block_at(s + 2);
                if (j2 >= 0)
                    issue_subtile<BLOCK, WAVES, KT, REMAP>(kbuf0, vbuf0, kpos0, buf, off, kr, j2, (s + 2) % SUBS,
                                                           j2 >= jmask, wave, lane);
            }
            fetch_rows(s + 3);
            {
                const int j = block_at(s + 1);
                if (j >= 0)
                    compute_subtile<BLOCK, NT, KT>(st, kbuf1, vbuf1, qf, qpos, kpos1,
                                               g.n - j * BLOCK - ((s + 1) % SUBS) * KT, j >= jmask, c2, ln, lh);
            }
        }
    }

    // ---- O' = diag(l)^-1 O; acc_o[dt][nt][x]: d = 32 dt + 8 (x / 4) + 4 h + (x % 4), query = q0 + 32 nt + n
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const float lt = st.l[nt] + __shfl_xor(st.l[nt], 32, 64);
        const float inv = lt > 0.0f ? 1.0f / lt : 0.0f;
        const int qs = q0 + 32 * nt + ln;
        if (qs < g.n) {
            bf16_t *dst = Op + ((size_t)bhq * g.n + qs) * D;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    floatx2 a = {st.acc_o[dt][nt][4 * gq] * inv, st.acc_o[dt][nt][4 * gq + 1] * inv};
                    floatx2 bb = {st.acc_o[dt][nt][4 * gq + 2] * inv, st.acc_o[dt][nt][4 * gq + 3] * inv};
                    const bf16x2 pa = __builtin_convertvector(a, bf16x2), pb = __builtin_convertvector(bb, bf16x2);
                    bf16x4 o4 = {pa[0], pa[1], pb[0], pb[1]};
                    *reinterpret_cast<bf16x4 *>(dst + 32 * dt + 8 * gq + 4 * lh) = o4;
                }
            if (lse && lh == 0)
                lse[(size_t)bhq * g.n + qs] = lt > 0.0f ? (st.mref[nt] + log2f(lt)) * kLn2F : -INFINITY;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Vector kernel: two threads per query row, each owning half of d.  K' and V'^T tiles are staged in LDS as
// fp32; every key updates the running (m, l, O) directly.  grid = (T, batch*h_q), 2*block threads.
// ---------------------------------------------------------------------------------------------
template <typename E, int D>
__global__ __launch_bounds__(256) void attn_vector_kernel(
    const E *__restrict__ Qp, const E *__restrict__ Kp, const E *__restrict__ Vt, const int32_t *__restrict__ qidx,
    const int32_t *__restrict__ kidx, const int32_t *__restrict__ row_cnt, const int32_t *__restrict__ col_idx,
    E *__restrict__ Op, float *__restrict__ lse, Geo g)
{
    constexpr int HALF = D / 2;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float *kt = reinterpret_cast<float *>(smem_raw);             // [block][D]
    float *vt = kt + g.block * D;                                // the block's Vt image: [block / G][D][G]
    int *kpos = reinterpret_cast<int *>(vt + D * g.block);       // [block]

    const int i = g.T - 1 - (int)blockIdx.x;
    const int bhq = blockIdx.y;
    const int b = bhq / g.h_q, hq = bhq % g.h_q;
    const size_t bhk = (size_t)b * g.h_kv + hq / g.r;
    const int row = threadIdx.x >> 1, half = threadIdx.x & 1;
    const int qs = i * g.block + row;
    const bool live = qs < g.n;
    const int qpos = live ? (qidx ? qidx[(size_t)bhq * g.n + qs] : qs) : -1;

    float q[HALF], o[HALF];
    {
        const E *src = Qp + ((size_t)bhq * g.n + (live ? qs : g.n - 1)) * D + half * HALF;
#pragma unroll
        for (int e = 0; e < HALF; ++e) { q[e] = ElemTraits<E>::to_float(src[e]); o[e] = 0.0f; }
    }
    float m = -INFINITY, l = 0.0f;
    const int ni = allowed_cols(i, g);
    const int cnt = min(row_cnt[(size_t)bhq * g.T + i], g.T);
    const int32_t *cols = col_idx + ((size_t)bhq * g.T + i) * g.T;
    const E *Kh = Kp + bhk * (size_t)g.n * D;
    const E *Vh = Vt + bhk * (size_t)g.T * D * g.block;
    const int32_t *kih = kidx + bhk * (size_t)g.n;
    const int G = vt_group(g.block);

    for (int t = 0; t < cnt; ++t) {
        const int j = cols[t];
        if (j < 0 || j >= ni) continue;
        __syncthreads();
        for (int c = threadIdx.x; c < g.block * D; c += blockDim.x) {
            const int kr = c / D, e = c % D;
            const int slot = j * g.block + kr;
            kt[c] = slot < g.n ? ElemTraits<E>::to_float(Kh[(size_t)slot * D + e]) : 0.0f;
            vt[c] = ElemTraits<E>::to_float(Vh[(size_t)j * D * g.block + c]);
        }
        for (int c = threadIdx.x; c < g.block; c += blockDim.x) {
            const int slot = j * g.block + c;
            kpos[c] = slot < g.n ? kih[slot] : INT_MAX;
        }
        __syncthreads();
        for (int c = 0; c < g.block; ++c) {
            float part = 0.0f;
            const float *kr = kt + c * D + half * HALF;
#pragma unroll
            for (int e = 0; e < HALF; ++e) part += q[e] * kr[e];
            const float s = (part + __shfl_xor(part, 1, 64)) * g.scale;
            if (kpos[c] > qpos) continue;
            if (s > m) {
                const float alpha = __expf(m - s);               // exp(-inf) = 0 on the first visible key
                l *= alpha;
#pragma unroll
                for (int e = 0; e < HALF; ++e) o[e] *= alpha;
                m = s;
            }
            const float p = __expf(s - m);
            l += p;
            const float *vr = vt + ((c / G) * D + half * HALF) * G + c % G;
#pragma unroll
            for (int e = 0; e < HALF; ++e) o[e] += p * vr[e * G];
        }
    }
    if (live) {
        const float inv = l > 0.0f ? 1.0f / l : 0.0f;
        E *dst = Op + ((size_t)bhq * g.n + qs) * D + half * HALF;
#pragma unroll
        for (int e = 0; e < HALF; ++e) dst[e] = ElemTraits<E>::from_float(o[e] * inv);
        if (lse && half == 0) lse[(size_t)bhq * g.n + qs] = l > 0.0f ? m + logf(l) : -INFINITY;
    }
}

// true when the 64-queries-per-wave kernel (attn_wide.hip) serves the problem
static bool wide_path(const pbs_problem *p) { return p->dtype == PBS_BF16 && p->d == 128 && p->block == 128; }

// The wide kernel leaves one flag per query block: blocks it could not finish with a fixed softmax reference.
size_t ws_attn_fwd(const pbs_problem *p)
{
    if (!wide_path(p)) return 0;
    const Geo g = make_geo(p);
    return align_up((size_t)g.batch * g.h_q * g.T * sizeof(int32_t), kWsAlign);
}

pbs_status launch_attn_wide(const Geo &g, const void *Qp, const void *Kp, const void *Vt, const int32_t *qidx,
                            const int32_t *kidx, const int32_t *row_cnt, const int32_t *col_idx, void *Op, float *lse,
                            int32_t *redo, int tok_delta, hipStream_t s);

template <typename E, int D>
static pbs_status launch_vector(const Geo &g, const void *Qp, const void *Kp, const void *Vt, const int32_t *qidx,
                                const int32_t *kidx, const int32_t *row_cnt, const int32_t *col_idx, void *Op,
                                float *lse, hipStream_t s)
{
    const size_t lds = (size_t)2 * g.block * D * sizeof(float) + (size_t)g.block * sizeof(int);
    static std::atomic<unsigned long long> lds_raised{0};
    if (lds > 32 * 1024) {
        const pbs_status st = raise_lds_limit(reinterpret_cast<const void *>(&attn_vector_kernel<E, D>),
                                              160 * 1024 - 2048, lds_raised);
        if (st != PBS_OK) return st;
    }
    return launch((attn_vector_kernel<E, D>), dim3(g.T, g.batch * g.h_q), dim3(2 * g.block), lds, s,
                       (const E *)Qp, (const E *)Kp, (const E *)Vt, qidx, kidx, row_cnt, col_idx, (E *)Op, lse, g);
}

}  // namespace pbs

using namespace pbs;

extern "C" pbs_status pbs_attn_fwd(const pbs_problem *p, const void *Qp, const void *Kp, const void *Vt,
                                   const int32_t *qidx, const int32_t *kidx, const int32_t *row_cnt,
                                   const int32_t *col_idx, void *Op, float *lse, void *ws, size_t ws_bytes,
                                   void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!Qp || !Kp || !Vt || !kidx || !row_cnt || !col_idx || !Op) return PBS_ERR_NULL;
    if (!aligned16(Qp) || !aligned16(Kp) || !aligned16(Vt) || !aligned16(Op)) return PBS_ERR_SHAPE;
    if ((st = check_ws(p, PBS_STAGE_ATTN_FWD, ws, ws_bytes)) != PBS_OK) return st;
    const Geo g = make_geo(p);
    hipStream_t s = (hipStream_t)stream;
    if (p->dtype == PBS_BF16 && p->d == 128 && (p->block == 128 || p->block == 64)) {
        const int ncoh = g.batch * g.h_kv * ((g.r * g.T + kCohort - 1) / kCohort);
        const dim3 mgrid((unsigned)(((ncoh + kXcds - 1) / kXcds) * kCohort * kXcds));
        const bool remap = (p->flags & PBS_FLAG_INDEX_REMAP) != 0;     // Kp is the caller's K
        const bool narrow_only = (p->flags & PBS_FLAG_RUNNING_MAX_ONLY) != 0 || remap;
        if (remap) {
            if (p->block == 128)
                return launch((attn_mfma_kernel<128, 4, 64, true>), mgrid, dim3(256), 0, s, (const bf16_t *)Qp,
                              (const bf16_t *)Kp, (const bf16_t *)Vt, qidx, kidx, row_cnt, col_idx, (bf16_t *)Op, lse,
                              (const int32_t *)nullptr, g);
            return launch((attn_mfma_kernel<64, 2, 32, true>), mgrid, dim3(128), 0, s, (const bf16_t *)Qp,
                          (const bf16_t *)Kp, (const bf16_t *)Vt, qidx, kidx, row_cnt, col_idx, (bf16_t *)Op, lse,
                          (const int32_t *)nullptr, g);
        }
        if (p->block == 128) {
            // first pass: every query block with a fixed softmax reference; second pass: the flagged blocks (none
            // on ordinary inputs, then each workgroup of the second launch leaves at once) with the rescaling kernel
            int32_t *redo = narrow_only ? nullptr : reinterpret_cast<int32_t *>(ws);
            if (redo) {
                // own segments from the token-order copies: identity sigma, and every byte of both copies of a head
                // within reach of 32-bit buffer offsets
                const long long tok_blocks = (long long)g.batch * g.h_kv * g.T;
                const bool own_tok = (p->flags & PBS_FLAG_TOKEN_ORDER_COPY) && !qidx &&
                                     (tok_blocks + g.T) * 128 * 256 < 0x7fffffffLL;
                const int tok_delta = own_tok ? (int)tok_blocks : 0;
                st = launch_attn_wide(g, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op, lse, redo, tok_delta, s);
                if (st != PBS_OK) return st;
            }
            st = launch((attn_mfma_kernel<128, 4, 64>), mgrid, dim3(256), 0, s, (const bf16_t *)Qp,
                               (const bf16_t *)Kp, (const bf16_t *)Vt, qidx, kidx, row_cnt, col_idx, (bf16_t *)Op, lse,
                               (const int32_t *)redo, g);
        } else {
            st = launch((attn_mfma_kernel<64, 2, 32>), mgrid, dim3(128), 0, s, (const bf16_t *)Qp,
                               (const bf16_t *)Kp, (const bf16_t *)Vt, qidx, kidx, row_cnt, col_idx, (bf16_t *)Op, lse,
                               (const int32_t *)nullptr, g);
        }
        return st;
    }
    if (p->flags & PBS_FLAG_INDEX_REMAP) return PBS_ERR_UNSUPPORTED;   // only the matrix-core kernels remap
    if (p->dtype == PBS_BF16)
        return p->d == 128 ? launch_vector<bf16_t, 128>(g, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op, lse, s)
                           : launch_vector<bf16_t, 64>(g, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op, lse, s);
    return p->d == 128 ? launch_vector<float, 128>(g, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op, lse, s)
                       : launch_vector<float, 64>(g, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op, lse, s);
}

