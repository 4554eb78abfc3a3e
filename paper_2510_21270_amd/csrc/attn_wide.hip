// pbs_attn_fwd for bf16, d = 128, block = 128: the "wide" matrix-core kernel of Algorithm 1's main loop.
//
// Same transposed formulation as the kernel in attn_fwd.hip (S^T = K' Q'^T, O^T += V'^T P^T, one lane owns one query
// of each 32-query tile), but every wave owns 64 queries (two 32-query tiles) and a workgroup is two waves, so that
// one wave runs per SIMD, and the softmax reference of a query is fixed at its first visible key (see kBigRowSum):
//   * every K' / V'^T fragment read from LDS feeds two MFMAs instead of one;
//   * the softmax arithmetic of a wave is interleaved, in its own instruction stream, with independent MFMAs (the
//     scores of the NEXT sub-tile, the O^T update of the other query tile), so the matrix pipe does not depend on a
//     second wave happening to be in the opposite phase.
// Key blocks are consumed in sub-tiles of 32 keys.  Sub-tile u of a list chunk covers keys [32 p, 32 p + 32),
// p = u % 4, of listed block u / 4 and lives in LDS stage p of a 4-deep ring filled by asynchronous buffer->LDS
// loads.  Iteration t:
//     X:  S(t + 1) MFMAs        || softmax(t) of query tile 0 || V'^T fragment reads of sub-tile t
//     Y:  O^T += ... tile 0     || softmax(t) of query tile 1 || K' fragment reads of sub-tile t + 2
//     Z:  O^T += ... tile 1     || barrier (every load issued so far has landed; stage t is free), then the
//                                  loads of sub-tile t + 4 into stage t
// A sub-tile that is not plain (token-level mask, queries without a visible key so far) first rewrites its scores
// and references in a separate block, then goes through the same groups.
#include "pbs_host.h"

namespace pbs {
namespace wide {

constexpr int BLOCK = 128, D = 128;
constexpr int KS = 32;                                     // keys per sub-tile
constexpr int kKRowB = 272;                                // K' row in LDS: 256 bytes + 16 of padding
constexpr int kVRowB = 80;                                 // V'^T row in LDS: 32 keys x 2 bytes + 16 of padding
constexpr int kKChunks = 9;                                // 32 x 272 = 8704 bytes -> nine 1 KiB load chunks
constexpr int kVChunks = 10;                               // 128 x 80 = 10240 bytes
constexpr int kLoadsPerWave = 10;                          // 16-byte-per-lane loads a wave issues per stage
constexpr int kList = 256;                                 // listed blocks staged in LDS at a time
constexpr int kXcds = 8, kCohort = 64;
constexpr float kLog2eF = 1.4426950408889634f;
constexpr float kLn2F = 0.6931471805599453f;
// The softmax reference of a query is the row maximum of the sub-tile that holds its first visible key and is never
// updated: any reference gives the same softmax as long as nothing overflows, and fp32 / bf16 have room for
// probabilities up to 2^64 relative to it (64 log2 units = 44 nats above the first sub-tile's maximum).  A partial
// row sum beyond that, infinite or NaN marks the whole query block as "bad"; the caller recomputes such blocks with
// the rescaling kernel.  This keeps every vector-ALU write away from the O^T accumulators.
constexpr float kBigRowSum = 1.8446744e19f;                // 2^64

typedef __attribute__((address_space(3))) void *lptr_t;

// One ring stage.  Each stage is a separate __shared__ variable so that the compiler can tell a fragment read of
// one stage from an asynchronous load into another.
struct __align__(16) Stage {
    unsigned char k[kKChunks * 1024];                      // row r holds key swap23(r) of the sub-tile
    unsigned char v[kVChunks * 1024];                      // row e holds V'^T[e][32 keys]
    int pos[64];                                           // original positions of the 32 keys (rest unused)
};

__device__ __forceinline__ int swap23(int m) { return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1); }

struct TileBuffers {
    __amdgpu_buffer_rsrc_t k, v, pos;
};

// The 19 chunks of a stage are loaded by the same ten instructions in both waves, with per-wave scalar operands:
// wave 0 takes the nine K' chunks and V'^T chunk 9, wave 1 takes V'^T chunks 0..8 (and chunk 8 once more, so that
// no branch on the wave index surrounds the instructions).  The 32 key positions ride on eight lanes of wave 0.
// o[c]: per-lane byte offset, inside one key block / one sub-tile, of what this lane moves in load c.
struct LaneOffsets {
    uint32_t o[kLoadsPerWave];
};

__device__ __forceinline__ uint32_t k_lane_offset(int chunk, int lane)
{
    const int pos = chunk * 1024 + lane * 16;
    const int row = pos / kKRowB, col = pos % kKRowB;
    return row < KS ? (uint32_t)(swap23(row) * 256 + (col < 256 ? col : 0)) : 0u;   // tail of chunk 8: padding
}

__device__ __forceinline__ uint32_t v_lane_offset(int chunk, int lane)
{
    const int pos = chunk * 1024 + lane * 16;
    const int row = pos / kVRowB, col = pos % kVRowB;
    return (uint32_t)(row * (BLOCK * 2) + (col < KS * 2 ? col : 0));
}

__device__ __forceinline__ LaneOffsets lane_offsets(int wave, int lane)
{
    LaneOffsets r;
#pragma unroll
    for (int c = 0; c < kKChunks; ++c) r.o[c] = wave == 0 ? k_lane_offset(c, lane) : v_lane_offset(c, lane);
    r.o[kKChunks] = v_lane_offset(wave == 0 ? 9 : 8, lane);
    return r;
}

// Scalar operands of the loads of part P of block j into stage sg.
struct StageLoad {
    __amdgpu_buffer_rsrc_t rsrc;       // loads 0..8
    int soff, soff_v, soff_pos;        // scalar byte offsets: loads 0..8, load 9 (always V'^T), positions
    unsigned char *dst, *dst9;         // LDS destinations of load 0 and of load 9
};

template <int P>
__device__ __forceinline__ StageLoad stage_load(Stage &sg, const TileBuffers &buf, int j, int wave)
{
    StageLoad a;
    const int slot0 = j * BLOCK + P * KS;
    a.soff_v = j * (D * BLOCK * 2) + P * (KS * 2);
    a.soff_pos = slot0 * 4;
    a.rsrc = wave == 0 ? buf.k : buf.v;
    a.soff = wave == 0 ? slot0 * 256 : a.soff_v;
    a.dst = wave == 0 ? sg.k : sg.v;
    a.dst9 = sg.v + (wave == 0 ? 9 : 8) * 1024;
    return a;
}

// load c of the ten
template <int C>
__device__ __forceinline__ void issue_load(const StageLoad &a, const TileBuffers &buf, const LaneOffsets &off)
{
    if (C < kKChunks) __builtin_amdgcn_raw_ptr_buffer_load_lds(a.rsrc, (lptr_t)(a.dst + C * 1024), 16, off.o[C], a.soff, 0, 0);
    else __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.v, (lptr_t)a.dst9, 16, off.o[kKChunks], a.soff_v, 0, 0);
}

// original positions of the sub-tile's 32 keys: 16 bytes on each of the first eight lanes of wave 0
__device__ __forceinline__ void issue_positions(Stage &sg, const StageLoad &a, const TileBuffers &buf, int wave, int lane)
{
    if (wave == 0 && lane < 8) __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.pos, (lptr_t)sg.pos, 16, lane * 16, a.soff_pos, 0, 0);
}

template <int P>
__device__ __forceinline__ void issue_stage(Stage &sg, const TileBuffers &buf, const LaneOffsets &off, int j, int wave,
                                            int lane)
{
    const StageLoad a = stage_load<P>(sg, buf, j, wave);
    issue_load<0>(a, buf, off); issue_load<1>(a, buf, off); issue_load<2>(a, buf, off); issue_load<3>(a, buf, off);
    issue_load<4>(a, buf, off); issue_load<5>(a, buf, off); issue_load<6>(a, buf, off); issue_load<7>(a, buf, off);
    issue_load<8>(a, buf, off); issue_load<9>(a, buf, off);
    issue_positions(sg, a, buf, wave, lane);
}

// Every asynchronous load of this wave has landed, then all waves meet: the stages loaded so far are complete.
__device__ __forceinline__ void sync_stages()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);                    // vmcnt(0), gfx9 encoding
    __syncthreads();
}

struct State {
    floatx16 acc_o[4][2];
    float mref[2], l[2];    // reference (log2 units) and sum of exp2(s*c2 - mref), this lane's half of the keys
    bool seen[2];           // the query has met a visible key, i.e. mref is set
    bool bad;               // a probability outgrew the fixed reference: this query block is redone by the caller
};

__device__ __forceinline__ void load_kf(bf16x8 (&kf)[8], const Stage &sg, int ln, int lh)
{
    const unsigned char *kl = sg.k + ln * kKRowB + lh * 16;
#pragma unroll
    for (int x = 0; x < 8; ++x) kf[x] = *reinterpret_cast<const bf16x8 *>(kl + x * 32);
}

__device__ __forceinline__ void load_vf(bf16x8 (&vf)[8], const Stage &sg, int ln, int lh)
{
    const unsigned char *vl = sg.v + ln * kVRowB + lh * 16;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2)
            vf[2 * dt + k2] = *reinterpret_cast<const bf16x8 *>(vl + dt * 32 * kVRowB + k2 * 32);
}

// Score MFMAs are written as assembly statements so that their operands sit where this kernel needs them: the
// result in vector registers (the softmax reads it there), the K' and Q' fragments in accumulation registers
// (AGPRs), which no other instruction of the loop needs (the Q' fragments of query tile 1 stay in vector registers to
// balance the two files).  Everything else is left to the compiler, whose MFMAs keep
// their accumulators -- O^T here -- in AGPRs.  The compiler does not see inside the statements, so the one software
// hazard of a matrix result that can occur is covered by hand: the scores are read by vector instructions, and that
// is always more than a dozen instructions after the last statement (next loop iteration) or behind mfma_fence().
template <int NT>
__device__ __forceinline__ void s_mfma_first(floatx16 &s, const bf16x8 &k, const bf16x8 &q)
{
    if (NT == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(s) : "a"(k), "a"(q));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "a"(k), "v"(q));
}
template <int NT>
__device__ __forceinline__ void s_mfma_next(floatx16 &s, const bf16x8 &k, const bf16x8 &q)
{
    if (NT == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "a"(k), "a"(q));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "a"(k), "v"(q));
}

// More wait states than the longest matrix-result hazard (18 after a 16-pass, 11 after an 8-pass instruction)
__device__ __forceinline__ void mfma_fence()
{
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
}

// S^T of one 32-key sub-tile for both query tiles.  s[nt][x]: key = 16 (x / 8) + 8 h + (x % 8), query = 32 nt + n.
__device__ __forceinline__ void s_mfma(floatx16 (&s)[2], const bf16x8 (&kf)[8], const bf16x8 (&qf)[2][8])
{
    s_mfma_first<0>(s[0], kf[0], qf[0][0]);
    s_mfma_first<1>(s[1], kf[0], qf[1][0]);
#pragma unroll
    for (int x = 1; x < 8; ++x) {
        s_mfma_next<0>(s[0], kf[x], qf[0][x]);
        s_mfma_next<1>(s[1], kf[x], qf[1][x]);
    }
}

// two probabilities: exp2(s * c2 - shift), packed; rsum += the rounded values
__device__ __forceinline__ bf16x2 exp2_pack2(float s0, float s1, float c2, float shift, float &rsum)
{
    floatx2 pr = {__builtin_amdgcn_exp2f(__builtin_fmaf(s0, c2, -shift)), __builtin_amdgcn_exp2f(__builtin_fmaf(s1, c2, -shift))};
    const bf16x2 t2 = __builtin_convertvector(pr, bf16x2);
    const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
    rsum = __builtin_amdgcn_fdot2_f32_bf16(t2, ones, rsum, false);
    return t2;
}

// What a sub-tile that is not plain needs before the softmax of one query tile: the token-level mask (masked scores
// become -inf, i.e. probability 0), and for queries that meet their first visible key the reference, set to the row
// maximum of this sub-tile.  A reference, once set, never moves (see the note on kBigRowSum), so O^T is never
// rescaled and the softmax itself is the same code for every sub-tile.
__device__ __forceinline__ void prepare_tile(State &st, int nt, floatx16 &s, const int *kpos, int room, bool masked,
                                             int qpos, float c2, int lh)
{
    if (masked) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int k8 = 16 * u + 8 * lh;                    // 8 consecutive keys of this lane
            const int4 a = *reinterpret_cast<const int4 *>(kpos + k8);
            const int4 b = *reinterpret_cast<const int4 *>(kpos + k8 + 4);
            const int kp[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            const int lim = room - k8;                         // keys x >= lim of this group do not exist
#pragma unroll
            for (int x = 0; x < 8; ++x)
                if (kp[x] > qpos || x >= lim) s[8 * u + x] = -INFINITY;
        }
    }
    if (!__all(st.seen[nt])) {
        float rmax = -INFINITY;
#pragma unroll
        for (int x = 0; x < 16; ++x) rmax = fmaxf(rmax, s[x]);
        rmax = fmaxf(rmax, __shfl_xor(rmax, 32, 64));
        const bool now = rmax != -INFINITY;
        if (!st.seen[nt]) st.mref[nt] = now ? rmax * c2 : 0.0f;
        st.seen[nt] = st.seen[nt] || now;
    }
}

// One iteration: sub-tile (block j, part P) is finished -- softmax and O^T update -- while the scores of the next
// sub-tile are formed.  s_cur: scores of this sub-tile (from the previous iteration); s_nxt: scores of the next one.
// kf holds the K' fragments of the next sub-tile on entry and those of the one after it on exit.
// sg_v: this sub-tile's stage (V'^T, positions); once every wave has read it (barrier after group Y) it receives
// part P of block j_load, four sub-tiles ahead.  sg_k: stage of the sub-tile after the next (K' fragments).
template <int P>
__device__ __forceinline__ void step(State &st, floatx16 (&s_cur)[2], floatx16 (&s_nxt)[2], bf16x8 (&kf)[8],
                                     const bf16x8 (&qf)[2][8], Stage &sg_v, const Stage &sg_k, const int (&qpos)[2],
                                     int room, bool masked, float c2, int ln, int lh, const TileBuffers &buf,
                                     const LaneOffsets &off, int j_load, int wave, int lane)
{
    bf16x8 vf[8], pf[2][2];
    if (masked || !__all(st.seen[0] && st.seen[1])) {
        asm volatile("" ::: "memory");                     // keeps this rare block out of the straight-line code
        prepare_tile(st, 0, s_cur[0], sg_v.pos, room, masked, qpos[0], c2, lh);
        prepare_tile(st, 1, s_cur[1], sg_v.pos, room, masked, qpos[1], c2, lh);
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- X (the score MFMAs are opaque statements, so the interleaving with the softmax of tile 0 is written out)
    const unsigned char *vl = sg_v.v + ln * kVRowB + lh * 16;
    float rsum0 = 0.0f;
    // The exponentials of pair x are issued in slot x, their pack and row sum in slot x + 1, so that no instruction
    // waits on the result of the one just before it.
    floatx2 pr0 = {0.0f, 0.0f}, ar0 = {0.0f, 0.0f};
#define PBS_PACK0(x)                                                                                         \
    {                                                                                                        \
        const bf16x2 t2 = __builtin_convertvector(pr0, bf16x2);                                              \
        const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};                                                    \
        rsum0 = __builtin_amdgcn_fdot2_f32_bf16(t2, ones, rsum0, false);                                     \
        pf[0][(x) >> 2][2 * ((x) & 3)] = t2[0];                                                              \
        pf[0][(x) >> 2][2 * ((x) & 3) + 1] = t2[1];                                                          \
    }
#define PBS_X_STEP(x)                                                                                        \
    {                                                                                                        \
        if ((x) == 0) {                                                                                      \
            s_mfma_first<0>(s_nxt[0], kf[0], qf[0][0]);                                                      \
            s_mfma_first<1>(s_nxt[1], kf[0], qf[1][0]);                                                      \
        } else {                                                                                             \
            s_mfma_next<0>(s_nxt[0], kf[x], qf[0][x]);                                                       \
            s_mfma_next<1>(s_nxt[1], kf[x], qf[1][x]);                                                       \
        }                                                                                                    \
        vf[x] = *reinterpret_cast<const bf16x8 *>(vl + ((x) >> 1) * 32 * kVRowB + ((x) & 1) * 32);           \
        if ((x) > 1) PBS_PACK0((x) - 2)                                                                      \
        if ((x) > 0) {                                                                                       \
            pr0[0] = __builtin_amdgcn_exp2f(ar0[0]);                                                         \
            pr0[1] = __builtin_amdgcn_exp2f(ar0[1]);                                                         \
        }                                                                                                    \
        ar0[0] = __builtin_fmaf(s_cur[0][2 * (x)], c2, -st.mref[0]);                                         \
        ar0[1] = __builtin_fmaf(s_cur[0][2 * (x) + 1], c2, -st.mref[0]);                                     \
        asm volatile("" : "+v"(pr0), "+v"(ar0));                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                                   \
    }
    PBS_X_STEP(0) PBS_X_STEP(1) PBS_X_STEP(2) PBS_X_STEP(3) PBS_X_STEP(4) PBS_X_STEP(5) PBS_X_STEP(6) PBS_X_STEP(7)
    PBS_PACK0(6)
    pr0[0] = __builtin_amdgcn_exp2f(ar0[0]);
    pr0[1] = __builtin_amdgcn_exp2f(ar0[1]);
    PBS_PACK0(7)
#undef PBS_PACK0
#undef PBS_X_STEP
    st.l[0] += rsum0;
    st.bad = st.bad || !(rsum0 <= kBigRowSum);
    // ---- Y: O^T update of tile 0 || softmax of tile 1 || K' fragments of the sub-tile after the next
    float rsum1 = 0.0f;
    const unsigned char *kl = sg_k.k + ln * kKRowB + lh * 16;
    // MFMA i of a group works on fragment PBS_MQ(i): the four O^T tiles with the first 16 keys, then with the other
    // 16, so that consecutive MFMAs never share an accumulator
#define PBS_MQ(i) ((((i) & 3) << 1) | ((i) >> 2))
    floatx2 pr1 = {0.0f, 0.0f}, ar1 = {0.0f, 0.0f};
#define PBS_PACK1(q)                                                                                         \
    {                                                                                                        \
        const bf16x2 t2 = __builtin_convertvector(pr1, bf16x2);                                              \
        const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};                                                    \
        rsum1 = __builtin_amdgcn_fdot2_f32_bf16(t2, ones, rsum1, false);                                     \
        pf[1][(q) >> 2][2 * ((q) & 3)] = t2[0];                                                              \
        pf[1][(q) >> 2][2 * ((q) & 3) + 1] = t2[1];                                                          \
    }
#define PBS_Y_STEP(q)                                                                                        \
    {                                                                                                        \
        st.acc_o[PBS_MQ(q) >> 1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                               \
            vf[PBS_MQ(q)], pf[0][PBS_MQ(q) & 1], st.acc_o[PBS_MQ(q) >> 1][0], 0, 0, 0);                      \
        kf[q] = *reinterpret_cast<const bf16x8 *>(kl + (q) * 32);                                            \
        if ((q) > 1) PBS_PACK1((q) - 2)                                                                      \
        if ((q) > 0) {                                                                                       \
            pr1[0] = __builtin_amdgcn_exp2f(ar1[0]);                                                         \
            pr1[1] = __builtin_amdgcn_exp2f(ar1[1]);                                                         \
        }                                                                                                    \
        ar1[0] = __builtin_fmaf(s_cur[1][2 * (q)], c2, -st.mref[1]);                                         \
        ar1[1] = __builtin_fmaf(s_cur[1][2 * (q) + 1], c2, -st.mref[1]);                                     \
        asm volatile("" : "+v"(pr1), "+v"(ar1));                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                                   \
    }
    PBS_Y_STEP(0) PBS_Y_STEP(1) PBS_Y_STEP(2) PBS_Y_STEP(3) PBS_Y_STEP(4) PBS_Y_STEP(5) PBS_Y_STEP(6) PBS_Y_STEP(7)
    PBS_PACK1(6)
    pr1[0] = __builtin_amdgcn_exp2f(ar1[0]);
    pr1[1] = __builtin_amdgcn_exp2f(ar1[1]);
    PBS_PACK1(7)
#undef PBS_PACK1
#undef PBS_Y_STEP
    st.l[1] += rsum1;
    st.bad = st.bad || !(rsum1 <= kBigRowSum);
    // ---- Z: O^T update of tile 1.  Two MFMAs are queued before the barrier, so the matrix pipe has work while the
    // waves meet; after the barrier every wave is done reading stage sg_v, which is refilled under the rest.
#define PBS_Z_MFMA(i)                                                                                        \
    st.acc_o[PBS_MQ(i) >> 1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                   \
        vf[PBS_MQ(i)], pf[1][PBS_MQ(i) & 1], st.acc_o[PBS_MQ(i) >> 1][1], 0, 0, 0);
    PBS_Z_MFMA(0) PBS_Z_MFMA(1)
    __builtin_amdgcn_sched_barrier(0);
    sync_stages();
    const StageLoad ld = stage_load<P>(sg_v, buf, j_load, wave);
    issue_load<0>(ld, buf, off); issue_load<1>(ld, buf, off);
    __builtin_amdgcn_sched_barrier(0);
    PBS_Z_MFMA(2)
    issue_load<2>(ld, buf, off); issue_load<3>(ld, buf, off);
    __builtin_amdgcn_sched_barrier(0);
    PBS_Z_MFMA(3)
    issue_load<4>(ld, buf, off); issue_load<5>(ld, buf, off);
    __builtin_amdgcn_sched_barrier(0);
    PBS_Z_MFMA(4)
    issue_load<6>(ld, buf, off); issue_load<7>(ld, buf, off);
    __builtin_amdgcn_sched_barrier(0);
    PBS_Z_MFMA(5)
    issue_load<8>(ld, buf, off); issue_load<9>(ld, buf, off);
    __builtin_amdgcn_sched_barrier(0);
    PBS_Z_MFMA(6)
    issue_positions(sg_v, ld, buf, wave, lane);
    __builtin_amdgcn_sched_barrier(0);
    PBS_Z_MFMA(7)
#undef PBS_Z_MFMA
#undef PBS_MQ
    __builtin_amdgcn_sched_barrier(0);
}

__global__ __launch_bounds__(128) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_wide_kernel(
    const bf16_t *__restrict__ Qp, const bf16_t *__restrict__ Kp, const bf16_t *__restrict__ Vt,
    const int32_t *__restrict__ qidx, const int32_t *__restrict__ kidx, const int32_t *__restrict__ row_cnt,
    const int32_t *__restrict__ col_idx, bf16_t *__restrict__ Op, float *__restrict__ lse,
    int32_t *__restrict__ redo, Geo g)
{
    __shared__ Stage sg0, sg1, sg2, sg3;                   // 4 x 19.25 KiB
    __shared__ int jl[kList];                              // listed blocks of the current chunk, -1 = not admissible
    __shared__ int bad_any;

    // Workgroup -> (query head, query block): cohorts of 64 rows of one kv head per XCD, longest lists first
    // (same decoding as the 32-queries-per-wave kernel).
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
    const size_t bhk = unit;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ln = lane & 31, lh = lane >> 5;
    const int q0 = i * BLOCK + wave * 64;
    const float c2 = g.scale * kLog2eF;

    // Q' fragments: lane (n, h) holds Q'[q0 + 32 nt + n][16 ks + 8 h .. +8]
    bf16x8 qf[2][8];
    int qpos[2];
    State st;
    st.bad = false;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int qs = q0 + 32 * nt + ln;
        const int qc = qs < g.n ? qs : g.n - 1;
        const bf16_t *src = Qp + ((size_t)bhq * g.n + qc) * D + 8 * lh;
#pragma unroll
        for (int k = 0; k < 8; ++k) qf[nt][k] = *reinterpret_cast<const bf16x8 *>(src + 16 * k);
        qpos[nt] = qs < g.n ? (qidx ? qidx[(size_t)bhq * g.n + qs] : qs) : -1;
        st.mref[nt] = 0.0f;
        st.l[nt] = 0.0f;
        st.seen[nt] = qs >= g.n;                  // padding rows never hold the wave on the careful path
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int x = 0; x < 16; ++x) st.acc_o[dt][nt][x] = 0.0f;
    }

    const int ni = allowed_cols(i, g);
    const int jmask = first_masked_col(i, g);
    const int cnt = min(row_cnt[(size_t)bhq * g.T + i], g.T);
    const int32_t *cols = col_idx + ((size_t)bhq * g.T + i) * g.T;
    constexpr int kRawDword = 0x00020000;                  // gfx9 descriptor word 3: raw 32-bit data format
    TileBuffers buf;
    buf.k = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(Kp + bhk * (size_t)g.n * D), 0, g.n * 256, kRawDword);
    buf.v = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(Vt + bhk * (size_t)g.T * D * BLOCK), 0,
                                              g.T * D * BLOCK * 2, kRawDword);
    buf.pos = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(kidx + bhk * (size_t)g.n), 0, g.n * 4, kRawDword);
    const LaneOffsets off = lane_offsets(wave, lane);

    // An entry that the causal structure does not admit is staged as -1: it is loaded as block 0 and processed as a
    // sub-tile with no existing key (room 0 on the exact path), which contributes nothing.
    auto entry = [&](int e) -> int { return __builtin_amdgcn_readfirstlane(jl[e]); };

    for (int base = 0; base < cnt; base += kList) {
        const int len = min(kList, cnt - base);
        __syncthreads();                                   // previous chunk fully consumed
        for (int t = threadIdx.x; t < len; t += 128) {
            const int j = cols[base + t];
            jl[t] = (j >= 0 && j < ni) ? j : -1;
        }
        __syncthreads();

        // prologue: the four parts of the first block, its first scores, the K' fragments of part 1
        int jraw = entry(0);
        int jc = jraw < 0 ? 0 : jraw;
        issue_stage<0>(sg0, buf, off, jc, wave, lane);
        issue_stage<1>(sg1, buf, off, jc, wave, lane);
        issue_stage<2>(sg2, buf, off, jc, wave, lane);
        issue_stage<3>(sg3, buf, off, jc, wave, lane);
        sync_stages();
        floatx16 sa[2], sb[2];
        bf16x8 kf[8];
        load_kf(kf, sg0, ln, lh);
        s_mfma(sa, kf, qf);
        mfma_fence();
        load_kf(kf, sg1, ln, lh);
        __builtin_amdgcn_sched_barrier(0);

        for (int e = 0; e < len; ++e) {
            const int enext = min(e + 1, len - 1);         // past the end: the last block again (results unused)
            const int jnraw = entry(enext);
            const int jn = jnraw < 0 ? 0 : jnraw;
            const bool masked = jraw < 0 || jraw >= jmask;
            const int room0 = jraw < 0 ? 0 : g.n - jraw * BLOCK;   // keys of the block that exist
            // part p: softmax and O^T update of part p; scores of part p + 1; K' fragments of part p + 2 (parts past
            // 3 are those of the next block); part p of the next block is loaded into the stage part p leaves
            step<0>(st, sa, sb, kf, qf, sg0, sg2, qpos, room0, masked, c2, ln, lh, buf, off, jn, wave, lane);
            step<1>(st, sb, sa, kf, qf, sg1, sg3, qpos, room0 - KS, masked, c2, ln, lh, buf, off, jn, wave, lane);
            step<2>(st, sa, sb, kf, qf, sg2, sg0, qpos, room0 - 2 * KS, masked, c2, ln, lh, buf, off, jn, wave, lane);
            step<3>(st, sb, sa, kf, qf, sg3, sg1, qpos, room0 - 3 * KS, masked, c2, ln, lh, buf, off, jn, wave, lane);
            jraw = jnraw;
            jc = jn;
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);                // the loads issued past the end have landed too
    }

    // redo[query block] = 1 when some probability outgrew its fixed reference (the caller recomputes the block)
    if (threadIdx.x == 0) bad_any = 0;
    __syncthreads();
    if (st.bad) bad_any = 1;
    __syncthreads();
    if (threadIdx.x == 0) redo[(size_t)bhq * g.T + i] = bad_any;

    // ---- O' = diag(l)^-1 O; acc_o[dt][nt][x]: d = 32 dt + 8 (x / 4) + 4 h + (x % 4), query = q0 + 32 nt + n
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
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

}  // namespace wide

// redo: [batch * h_q * T] flags, written for every query block.
pbs_status launch_attn_wide(const Geo &g, const void *Qp, const void *Kp, const void *Vt, const int32_t *qidx,
                            const int32_t *kidx, const int32_t *row_cnt, const int32_t *col_idx, void *Op, float *lse,
                            int32_t *redo, hipStream_t s)
{
    const int ncoh = g.batch * g.h_kv * ((g.r * g.T + wide::kCohort - 1) / wide::kCohort);
    const dim3 grid((unsigned)(((ncoh + wide::kXcds - 1) / wide::kXcds) * wide::kCohort * wide::kXcds));
    hipLaunchKernelGGL(wide::attn_wide_kernel, grid, dim3(128), 0, s, (const bf16_t *)Qp, (const bf16_t *)Kp,
                       (const bf16_t *)Vt, qidx, kidx, row_cnt, col_idx, (bf16_t *)Op, lse, redo, g);
    return launch_status();
}

}  // namespace pbs
