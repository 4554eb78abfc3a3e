// pbs_attn_fwd for bf16, d = 128, block = 128: the "wide" matrix-core kernel of Algorithm 1's main loop.
//
// Same transposed formulation as the kernel in attn_fwd.hip (S^T = K' Q'^T, O^T += V'^T P^T, one lane owns one query
// of each 32-query tile), but every wave owns 64 queries (two 32-query tiles) and a workgroup is two waves, so that
// one wave runs per SIMD, and the softmax reference of a query is fixed at its first visible key (see kBigRowSum):
//   * every K' / V'^T fragment read from LDS feeds two MFMAs instead of one;
//   * the softmax arithmetic of a wave is interleaved, in its own instruction stream, with independent MFMAs (the
//     scores of the NEXT sub-tile, the O^T update with the PREVIOUS one), so the matrix pipe does not depend on a
//     second wave happening to be in the opposite phase.
// Key blocks are consumed in sub-tiles of 32 keys.  Sub-tile u of a list chunk covers keys [32 p, 32 p + 32),
// p = u % 4, of listed block u / 4.  A wave has a single instruction stream to itself, so the loop is a three-deep
// software pipeline in which no MFMA of an iteration depends on the vector arithmetic of the same iteration, and that
// arithmetic is spread evenly over the iteration's 32 MFMAs.  Iteration t:
//     MFMAs  0..15:  S(t + 1) = K'(t + 1) Q'^T, both query tiles
//     MFMAs 16..31:  O^T += V'^T(t - 1) P^T(t - 1), both query tiles
//     all along:     P^T(t) = softmax arithmetic on S(t), one score pair per two MFMAs
//     LDS traffic:   V'^T(t - 1) fragment reads under MFMAs 0..7; after MFMA 11 the waves meet (every load issued
//                    two or more iterations ago has landed, the V'^T part just read is free); the loads of K'(t + 4),
//                    V'^T(t + 3) and the key positions of sub-tile t + 4 go out under MFMAs 12..20; K'(t + 2)
//                    fragment reads under MFMAs 16..23
// LDS holds a 4-deep ring of stages filled by asynchronous buffer->LDS loads; stage p holds the K' part p and the
// V'^T part (p + 3) % 4 of their blocks, which is what iteration t = p (mod 4) frees and refills.
// A sub-tile that is not plain (token-level mask, queries without a visible key so far) first rewrites its scores
// and references in a separate block, then goes through the same code.
// The block list of a query block is staged in LDS in chunks, each entry as (block to load, keys that exist, mask
// bit).  When K', Vt and kidx carry a token-order copy behind the permuted tensors (tok_delta > 0), the R own-segment
// blocks at the end of a list are replaced, while staged, by the token-order blocks up to the diagonal; the loop
// itself does not know the difference (a token-order block is just a block index beyond the permuted ones).
#include "pbs_host.h"

namespace pbs {
namespace wide {

constexpr int BLOCK = 128, D = 128;
constexpr int KS = 32;                                     // keys per sub-tile
constexpr int kStageB = 8192;                              // K' sub-tile: 32 rows x 256 B; V'^T sub-tile: 128 rows x 64 B
constexpr int kLoadsPerWave = 8;                           // 16-byte-per-lane loads a wave issues per stage
constexpr int kList = 1024;                                // listed blocks staged in LDS at a time
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
// one stage from an asynchronous load into another.  Rows are not padded; instead the 16-byte pieces of a row are
// stored XOR-permuted so that the fragment reads below (16 lanes = 16 rows at one logical column) fall into 16
// different bank groups:
//   k: row r (256 B) holds key swap23(r) of the sub-tile, its logical piece c (of 16) at place c ^ (r % 16);
//   v: row e (64 B) holds V'^T[e][32 keys], its logical piece c (of 4) at place c ^ ((e / 4) % 4).
struct __align__(16) Stage {
    unsigned char k[kStageB];
    unsigned char v[kStageB];
    int pos[2 * KS];                                       // original positions of the keys in k (and of the next 32)
};

__device__ __forceinline__ int swap23(int m) { return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1); }

struct TileBuffers {
    __amdgpu_buffer_rsrc_t k, v, pos;
};

// A stage is 16 chunks of 1 KiB, one load instruction each (64 lanes x 16 bytes, consecutive in LDS).  Both waves
// execute the same eight instructions with per-wave operands: wave 0 brings the K' sub-tile, wave 1 the V'^T one.
// dma[c]: byte offset inside one key block (K': inside the sub-tile) of the piece this lane moves in load c.
// kfr[x], vfr[k2]: byte offsets inside a stage's k / v array of this lane's fragment reads.
struct LaneOffsets {
    uint32_t dma[kLoadsPerWave];
    uint32_t kfr[8], vfr[2];
};

__device__ __forceinline__ uint32_t k_lane_offset(int chunk, int lane)
{
    const int row = chunk * 4 + (lane >> 4), place = lane & 15;
    return (uint32_t)(swap23(row) * 256 + ((place ^ (row & 15)) << 4));
}

// Vt keeps a block as four groups of 32 keys, each [128 features][32 keys]: a sub-tile is 8 KiB of consecutive bytes
__device__ __forceinline__ uint32_t v_lane_offset(int chunk, int lane)
{
    const int row = chunk * 16 + (lane >> 2), place = lane & 3;
    return (uint32_t)(row * (KS * 2) + ((place ^ ((row >> 2) & 3)) << 4));
}

__device__ __forceinline__ LaneOffsets lane_offsets(int wave, int lane)
{
    LaneOffsets r;
    const int ln = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int c = 0; c < kLoadsPerWave; ++c) r.dma[c] = wave == 0 ? k_lane_offset(c, lane) : v_lane_offset(c, lane);
    // K' fragment x: logical piece 2 x + h of row n;  V'^T fragment (dt, k2): logical piece 2 k2 + h of row 32 dt + n
#pragma unroll
    for (int x = 0; x < 8; ++x) r.kfr[x] = (uint32_t)(ln * 256 + (((2 * x + lh) ^ (ln & 15)) << 4));
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) r.vfr[k2] = (uint32_t)(ln * 64 + (((2 * k2 + lh) ^ ((ln >> 2) & 3)) << 4));
    return r;
}

// Scalar operands of the loads of part P of block j into stage sg.
struct StageLoad {
    __amdgpu_buffer_rsrc_t rsrc;
    int soff;                          // scalar byte offset of the sub-tile in the tensor
    unsigned char *dst;                // LDS destination of load 0
};

// Stage P receives the K' part P of block jk and the V'^T part (P + 3) % 4 of block jv.
template <int P>
__device__ __forceinline__ StageLoad stage_load(Stage &sg, const TileBuffers &buf, int jk, int jv, int wave)
{
    StageLoad a;
    a.rsrc = wave == 0 ? buf.k : buf.v;
    a.soff = wave == 0 ? (jk * BLOCK + P * KS) * 256 : jv * (D * BLOCK * 2) + ((P + 3) & 3) * (D * KS * 2);
    a.dst = wave == 0 ? sg.k : sg.v;
    return a;
}

// load c of the eight
template <int C>
__device__ __forceinline__ void issue_load(const StageLoad &a, const LaneOffsets &off)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(a.rsrc, (lptr_t)(a.dst + C * 1024), 16, off.dma[C], a.soff, 0, 0);
}

// Original positions of the 32 keys of part P of block j, next to their K' rows.  Only sub-tiles under the
// token-level mask read them, but the load is issued for every sub-tile, by all lanes of both waves (four bytes per
// lane, the same 256 bytes from each wave): one more instruction in the stream costs less than a branch around it.
template <int P>
__device__ __forceinline__ void issue_positions(Stage &sg, const TileBuffers &buf, int j, int lane)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.pos, (lptr_t)sg.pos, 4, lane * 4, (j * BLOCK + P * KS) * 4, 0, 0);
}

template <int P>
__device__ __forceinline__ void issue_stage(Stage &sg, const TileBuffers &buf, const LaneOffsets &off, int j, int wave,
                                            int lane)
{
    const StageLoad a = stage_load<P>(sg, buf, j, j, wave);
    issue_load<0>(a, off); issue_load<1>(a, off); issue_load<2>(a, off); issue_load<3>(a, off);
    issue_load<4>(a, off); issue_load<5>(a, off); issue_load<6>(a, off); issue_load<7>(a, off);
    issue_positions<P>(sg, buf, j, lane);
}

// Every asynchronous load of this wave has landed, then all waves meet: the stages loaded so far are complete.
__device__ __forceinline__ void sync_stages()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);                    // vmcnt(0), gfx9 encoding
    __syncthreads();
}

// The loop's meeting point.  Each wave has waited for all of its loads except the nine it issued in the previous
// iteration, and for its fragment reads; after the barrier the loads of every wave up to two iterations back are
// complete.  That is all an iteration needs: it reads K' fragments loaded two iterations earlier and V'^T fragments
// loaded four iterations earlier, so a load has two full iterations to arrive.  (A plain barrier instruction, not
// __syncthreads(): the fence of the latter would wait for every load.)
__device__ __forceinline__ void sync_older_stages()
{
    __builtin_amdgcn_s_waitcnt(0x0079);                    // vmcnt(9) lgkmcnt(0), gfx9 encoding
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

struct State {
    floatx16 acc_o[4][2];
    float mref[2], l[2];    // reference (log2 units) and sum of exp2(s*c2 - mref), this lane's half of the keys
    bool seen[2];           // the query has met a visible key, i.e. mref is set
    bool bad;               // a probability outgrew the fixed reference: this query block is redone by the caller
};

__device__ __forceinline__ void load_kf(bf16x8 (&kf)[8], const Stage &sg, const LaneOffsets &off)
{
#pragma unroll
    for (int x = 0; x < 8; ++x) kf[x] = *reinterpret_cast<const bf16x8 *>(sg.k + off.kfr[x]);
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

// What a sub-tile that is not plain needs before the softmax of one query tile: the token-level mask (masked scores
// become -inf, i.e. probability 0), and for queries that meet their first visible key the reference, set to the row
// maximum of this sub-tile.  A reference, once set, never moves (see the note on kBigRowSum), so O^T is never
// rescaled and the softmax itself is the same code for every sub-tile.
__device__ __forceinline__ void mask_tile(floatx16 (&s)[2], const int *kpos, int room, const int (&qpos)[2], int lh)
{
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int k8 = 16 * u + 8 * lh;                        // 8 consecutive keys of this lane
        // original positions of the keys; slots past the end of the sequence hold 0 and are masked by lim
        const int4 a = *reinterpret_cast<const int4 *>(kpos + k8);
        const int4 b = *reinterpret_cast<const int4 *>(kpos + k8 + 4);
        const int kp[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        if (room >= KS) {                                      // every key of the sub-tile exists (all but a ragged tail)
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                if (kp[x] > qpos[0]) s[0][8 * u + x] = -INFINITY;
                if (kp[x] > qpos[1]) s[1][8 * u + x] = -INFINITY;
            }
        } else {
            const int lim = room - k8;                         // keys x >= lim of this group do not exist
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                if (kp[x] > qpos[0] || x >= lim) s[0][8 * u + x] = -INFINITY;
                if (kp[x] > qpos[1] || x >= lim) s[1][8 * u + x] = -INFINITY;
            }
        }
    }
}

__device__ __forceinline__ void set_reference(State &st, int nt, const floatx16 &s, float c2)
{
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

// One iteration t (t = P mod 4) of the pipeline described at the top of the file.
// s_cur: scores of sub-tile t (formed by the previous iteration); s_nxt: receives the scores of sub-tile t + 1.
// kf: K' fragments of sub-tile t + 1 on entry, of sub-tile t + 2 on exit.
// pf_prev: probabilities of sub-tile t - 1 (from the previous iteration); pf_new: receives those of sub-tile t.
// sg_v: stage P, whose V'^T part belongs to sub-tile t - 1; after the barrier it receives the K' part P of block jk
// and the V'^T part (P + 3) % 4 of block jv.  sg_k: stage (P + 2) % 4, K' fragments of sub-tile t + 2.
// room / masked describe sub-tile t (its key positions are in sg_v.pos).
template <int P>
__device__ __forceinline__ void step(State &st, floatx16 (&s_cur)[2], floatx16 (&s_nxt)[2], bf16x8 (&kf)[8],
                                     const bf16x8 (&qf)[2][8], const bf16x8 (&pf_prev)[2][2], bf16x8 (&pf_new)[2][2],
                                     Stage &sg_v, const Stage &sg_k, const int (&qpos)[2], int room, bool masked,
                                     float c2, int lh, const TileBuffers &buf, const LaneOffsets &off, int jk, int jv,
                                     int wave, int lane)
{
    bf16x8 vf[8];
    if (masked || !__all(st.seen[0] && st.seen[1])) {
        asm volatile("" ::: "memory");                     // keeps this rare block out of the straight-line code
        if (masked) mask_tile(s_cur, sg_v.pos, room, qpos, lh);
        set_reference(st, 0, s_cur[0], c2);
        set_reference(st, 1, s_cur[1], c2);
    }
    __builtin_amdgcn_sched_barrier(0);
    // Softmax of score pair q (query tile q / 8, scores 2 (q % 8) and + 1) in three stages, issued in consecutive
    // MFMA slots so that no instruction waits on the one just before it: multiply-add in slot 2 q, exponentials in
    // slot 2 q + 1, rounding / row sum / pack in slot 2 q + 2.  The row sum adds the unrounded probabilities with two
    // plain additions: on this chip the bf16 dot-product instruction that would sum the rounded pair in one go does
    // not overlap with the matrix instructions the way ordinary vector arithmetic does.
    floatx2 rsum[2] = {{0.0f, 0.0f}, {0.0f, 0.0f}};        // per query tile: sums over even and odd scores
    floatx2 pr = {0.0f, 0.0f}, ar = {0.0f, 0.0f};
#define PBS_SM_FMA(q)                                                                                        \
    {                                                                                                        \
        ar[0] = __builtin_fmaf(s_cur[(q) >> 3][2 * ((q) & 7)], c2, -st.mref[(q) >> 3]);                      \
        ar[1] = __builtin_fmaf(s_cur[(q) >> 3][2 * ((q) & 7) + 1], c2, -st.mref[(q) >> 3]);                  \
    }
#define PBS_SM_EXP(q)                                                                                        \
    {                                                                                                        \
        pr[0] = __builtin_amdgcn_exp2f(ar[0]);                                                               \
        pr[1] = __builtin_amdgcn_exp2f(ar[1]);                                                               \
    }
#define PBS_SM_PACK(q)                                                                                       \
    {                                                                                                        \
        bf16x2 t2 = __builtin_convertvector(pr, bf16x2);                                                     \
        asm volatile("" : "+v"(t2));                       /* the pack happens here, not where it is consumed */ \
        rsum[(q) >> 3] += pr;                                                                                \
        asm volatile("" : "+v"(rsum[(q) >> 3]));                                                             \
        pf_new[(q) >> 3][((q) & 7) >> 2][2 * ((q) & 3)] = t2[0];                                             \
        pf_new[(q) >> 3][((q) & 7) >> 2][2 * ((q) & 3) + 1] = t2[1];                                         \
    }
    // vector work of MFMA slot m
#define PBS_SM_SLOT(m)                                                                                       \
    {                                                                                                        \
        if (((m) & 1) == 0) {                                                                                \
            if ((m) > 0) PBS_SM_PACK((((m) >> 1) + 15) & 15)                                                 \
            PBS_SM_FMA((m) >> 1)                                                                             \
        } else {                                                                                             \
            PBS_SM_EXP((m) >> 1)                                                                             \
        }                                                                                                    \
        asm volatile("" : "+v"(pr), "+v"(ar));                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                                   \
    }
    // ---- slots 0..15: score MFMAs of sub-tile t + 1 (opaque statements, so the interleaving is written out).
    // The V'^T fragments are read in slots 0..7.  After slot 11 the waves meet: every wave has those fragments in
    // registers (stage sg_v is free) and every load issued so far has landed; the refill of sg_v is issued under
    // slots 12..19.  K' fragment reads of sub-tile t + 2 take slots 16..23.
#define PBS_S_MFMA(m)                                                                                        \
    {                                                                                                        \
        if ((m) == 0) s_mfma_first<0>(s_nxt[0], kf[0], qf[0][0]);                                            \
        else if ((m) == 1) s_mfma_first<1>(s_nxt[1], kf[0], qf[1][0]);                                       \
        else if (((m) & 1) == 0) s_mfma_next<0>(s_nxt[0], kf[(m) >> 1], qf[0][(m) >> 1]);                    \
        else s_mfma_next<1>(s_nxt[1], kf[(m) >> 1], qf[1][(m) >> 1]);                                        \
        asm volatile("" : "+v"(pr), "+v"(ar));             /* the slot's vector work follows its MFMA */     \
    }
#define PBS_VF_SLOT(m)                                                                                       \
    {                                                                                                        \
        PBS_S_MFMA(m)                                                                                        \
        vf[m] = *reinterpret_cast<const bf16x8 *>(sg_v.v + off.vfr[(m) & 1] + ((m) >> 1) * 2048);            \
        PBS_SM_SLOT(m)                                                                                       \
    }
#define PBS_S_SLOT(m)                                                                                        \
    {                                                                                                        \
        PBS_S_MFMA(m)                                                                                        \
        PBS_SM_SLOT(m)                                                                                       \
    }
#define PBS_SLD_SLOT(m)                                                                                      \
    {                                                                                                        \
        PBS_S_MFMA(m)                                                                                        \
        issue_load<(m) - 12>(ld, off);                                                                       \
        PBS_SM_SLOT(m)                                                                                       \
    }
    PBS_VF_SLOT(0) PBS_VF_SLOT(1) PBS_VF_SLOT(2) PBS_VF_SLOT(3) PBS_VF_SLOT(4) PBS_VF_SLOT(5) PBS_VF_SLOT(6) PBS_VF_SLOT(7)
    PBS_S_SLOT(8) PBS_S_SLOT(9) PBS_S_SLOT(10) PBS_S_SLOT(11)
    sync_older_stages();
    const StageLoad ld = stage_load<P>(sg_v, buf, jk, jv, wave);
    PBS_SLD_SLOT(12) PBS_SLD_SLOT(13) PBS_SLD_SLOT(14) PBS_SLD_SLOT(15)
#undef PBS_SLD_SLOT
#undef PBS_S_SLOT
#undef PBS_VF_SLOT
#undef PBS_S_MFMA
    // ---- slots 16..31: O^T update with sub-tile t - 1.  MFMA i of a query tile works on fragment PBS_MQ(i): the four
    // O^T tiles with the first 16 keys, then with the other 16, so that consecutive MFMAs never share an accumulator.
#define PBS_MQ(i) ((((i) & 3) << 1) | ((i) >> 2))
#define PBS_PV_MFMA(n)                                                                                       \
    st.acc_o[PBS_MQ((n) & 7) >> 1][(n) >> 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                      \
        vf[PBS_MQ((n) & 7)], pf_prev[(n) >> 3][PBS_MQ((n) & 7) & 1], st.acc_o[PBS_MQ((n) & 7) >> 1][(n) >> 3], 0, 0, 0);
#define PBS_KF_READ(n) kf[n] = *reinterpret_cast<const bf16x8 *>(sg_k.k + off.kfr[n]);
#define PBS_PLD_SLOT(n)                                                                                      \
    {                                                                                                        \
        PBS_PV_MFMA(n)                                                                                       \
        issue_load<(n) + 4>(ld, off);                                                                        \
        PBS_KF_READ(n)                                                                                       \
        PBS_SM_SLOT(16 + (n))                                                                                \
    }
#define PBS_KF_SLOT(n)                                                                                       \
    {                                                                                                        \
        PBS_PV_MFMA(n)                                                                                       \
        PBS_KF_READ(n)                                                                                       \
        PBS_SM_SLOT(16 + (n))                                                                                \
    }
#define PBS_PV_SLOT(n)                                                                                       \
    {                                                                                                        \
        PBS_PV_MFMA(n)                                                                                       \
        PBS_SM_SLOT(16 + (n))                                                                                \
    }
    PBS_PLD_SLOT(0) PBS_PLD_SLOT(1) PBS_PLD_SLOT(2) PBS_PLD_SLOT(3)
    issue_positions<P>(sg_v, buf, jk, lane);
    PBS_KF_SLOT(4) PBS_KF_SLOT(5) PBS_KF_SLOT(6) PBS_KF_SLOT(7)
    PBS_PV_SLOT(8) PBS_PV_SLOT(9) PBS_PV_SLOT(10) PBS_PV_SLOT(11) PBS_PV_SLOT(12) PBS_PV_SLOT(13) PBS_PV_SLOT(14)
    PBS_PV_SLOT(15)
    PBS_SM_PACK(15)
#undef PBS_PV_SLOT
#undef PBS_KF_SLOT
#undef PBS_PLD_SLOT
#undef PBS_KF_READ
#undef PBS_PV_MFMA
#undef PBS_SM_SLOT
#undef PBS_SM_PACK
#undef PBS_SM_EXP
#undef PBS_SM_FMA
    const float rs0 = rsum[0][0] + rsum[0][1], rs1 = rsum[1][0] + rsum[1][1];
    st.l[0] += rs0;
    st.l[1] += rs1;
    st.bad = st.bad || !(rs0 <= kBigRowSum) || !(rs1 <= kBigRowSum);
    __builtin_amdgcn_sched_barrier(0);
}

// End of a list chunk: the O^T update with its last sub-tile (part 3 of the last block, in stage 0).
__device__ __forceinline__ void drain(State &st, const bf16x8 (&pf)[2][2], const Stage &sg, const LaneOffsets &off)
{
    bf16x8 vf[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) vf[x] = *reinterpret_cast<const bf16x8 *>(sg.v + off.vfr[x & 1] + (x >> 1) * 2048);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 8; ++i)
            st.acc_o[PBS_MQ(i) >> 1][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                vf[PBS_MQ(i)], pf[nt][PBS_MQ(i) & 1], st.acc_o[PBS_MQ(i) >> 1][nt], 0, 0, 0);
}
#undef PBS_MQ

__global__ __launch_bounds__(128) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_wide_kernel(
    const bf16_t *__restrict__ Qp, const bf16_t *__restrict__ Kp, const bf16_t *__restrict__ Vt,
    const int32_t *__restrict__ qidx, const int32_t *__restrict__ kidx, const int32_t *__restrict__ row_cnt,
    const int32_t *__restrict__ col_idx, bf16_t *__restrict__ Op, float *__restrict__ lse,
    int32_t *__restrict__ redo, Geo g, int tok_delta)
{
    __shared__ Stage sg0, sg1, sg2, sg3;                   // 4 x 16 KiB
    __shared__ int jl[kList];                              // current chunk of the list: block index to load
    __shared__ int jm[kList];                              // ... keys of that block that exist, bit 30: token-level mask
    __shared__ int bad_any;
    __shared__ int own_tail_ok;                            // the chunk ends with the whole own segment, ascending

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
    // tok_delta > 0: a token-order copy of K', Vt and kidx lies tok_delta = batch * h_kv * T blocks behind the
    // permuted one, so block j of this head in token order is block tok_delta + j of the same descriptors
    const int reach = tok_delta * BLOCK + g.n;             // rows within reach of this head's descriptors
    buf.k = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(Kp + bhk * (size_t)g.n * D), 0, reach * 256, kRawDword);
    buf.v = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(Vt + bhk * (size_t)g.T * D * BLOCK), 0,
                                              (tok_delta + g.T) * (D * BLOCK * 2), kRawDword);
    buf.pos = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(kidx + bhk * (size_t)g.n), 0, reach * 4, kRawDword);
    const LaneOffsets off = lane_offsets(wave, lane);

    // The list is staged as (block to load, keys that exist | mask bit).  An entry that the causal structure does not
    // admit is staged as block 0 with no existing key and the mask bit: a sub-tile that contributes nothing.
    constexpr int kMaskBit = 1 << 30;
    auto entry = [&](int e) -> int { return __builtin_amdgcn_readfirstlane(jl[e]); };
    auto entry_meta = [&](int e) -> int { return __builtin_amdgcn_readfirstlane(jm[e]); };

    for (int base = 0; base < cnt; base += kList) {
        int len = min(kList, cnt - base);
        __syncthreads();                                   // previous chunk fully consumed
        if (threadIdx.x == 0) own_tail_ok = 1;
        for (int t = threadIdx.x; t < len; t += 128) {
            const int j = cols[base + t];
            const bool ok = j >= 0 && j < ni;
            jl[t] = ok ? j : 0;
            jm[t] = ok ? (g.n - j * BLOCK) | (j >= jmask ? kMaskBit : 0) : kMaskBit;
        }
        __syncthreads();
        // Own segment in token order: when the list ends with all blocks jmask .. ni - 1 of the query block's own
        // (full) segment, ascending, they are replaced by the blocks jmask .. i of the token-order copies.
        // Keys of a segment are the same set in either order, so the visible keys are the same; in token order
        // the blocks before the diagonal need no mask and those after it hold no visible key.
        if (tok_delta > 0 && i / g.R < g.G && base + len == cnt && len >= ni - jmask) {
            const int own = ni - jmask, first = len - own;
            const int t = threadIdx.x;
            if (t < own && (jl[first + t] != jmask + t || jm[first + t] != ((g.n - (jmask + t) * BLOCK) | kMaskBit)))
                own_tail_ok = 0;
            __syncthreads();
            if (own_tail_ok) {
                if (t <= i - jmask) {
                    jl[first + t] = tok_delta + jmask + t;
                    jm[first + t] = (g.n - (jmask + t) * BLOCK) | (jmask + t == i ? kMaskBit : 0);
                }
                len = first + i - jmask + 1;
            }
            __syncthreads();
        }

        // prologue: the four parts of the first block, its first scores, the K' fragments of part 1
        int jc = entry(0);
        int meta = entry_meta(0);
        issue_stage<0>(sg0, buf, off, jc, wave, lane);
        issue_stage<1>(sg1, buf, off, jc, wave, lane);
        issue_stage<2>(sg2, buf, off, jc, wave, lane);
        issue_stage<3>(sg3, buf, off, jc, wave, lane);
        sync_stages();
        floatx16 sa[2], sb[2];
        bf16x8 kf[8];
        load_kf(kf, sg0, off);
        s_mfma(sa, kf, qf);
        mfma_fence();
        load_kf(kf, sg1, off);
        bf16x8 pa[2][2], pb[2][2];                         // probabilities of the previous / the current sub-tile
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int x = 0; x < 8; ++x) pa[u >> 1][u & 1][x] = (bf16_t)0.0f;
        __builtin_amdgcn_sched_barrier(0);

        for (int e = 0; e < len; ++e) {
            const int enext = min(e + 1, len - 1);         // past the end: the last block again (results unused)
            const int jn = entry(enext);
            const int meta_next = entry_meta(enext);
            const bool masked = (meta & kMaskBit) != 0;
            const int room0 = meta & (kMaskBit - 1);       // keys of the block that exist
            // part p: probabilities of part p; scores of part p + 1; O^T update with part p - 1; K' fragments of
            // part p + 2 (parts outside 0..3 are those of the neighbouring listed blocks).  Stage p is refilled with
            // K' part p of the next block and V'^T part p - 1 of the next block (part 3 of this block when p = 0).
            // The first iteration of a chunk updates O^T with zero probabilities.
            step<0>(st, sa, sb, kf, qf, pa, pb, sg0, sg2, qpos, room0, masked, c2, lh, buf, off, jn, jc, wave, lane);
            step<1>(st, sb, sa, kf, qf, pb, pa, sg1, sg3, qpos, room0 - KS, masked, c2, lh, buf, off, jn, jn, wave, lane);
            step<2>(st, sa, sb, kf, qf, pa, pb, sg2, sg0, qpos, room0 - 2 * KS, masked, c2, lh, buf, off, jn, jn, wave, lane);
            step<3>(st, sb, sa, kf, qf, pb, pa, sg3, sg1, qpos, room0 - 3 * KS, masked, c2, lh, buf, off, jn, jn, wave, lane);
            jc = jn;
            meta = meta_next;
        }
        drain(st, pa, sg0, off);
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
                            int32_t *redo, int tok_delta, hipStream_t s)
{
    const int ncoh = g.batch * g.h_kv * ((g.r * g.T + wide::kCohort - 1) / wide::kCohort);
    const dim3 grid((unsigned)(((ncoh + wide::kXcds - 1) / wide::kXcds) * wide::kCohort * wide::kXcds));
    return launch(wide::attn_wide_kernel, grid, dim3(128), 0, s, (const bf16_t *)Qp, (const bf16_t *)Kp,
                       (const bf16_t *)Vt, qidx, kidx, row_cnt, col_idx, (bf16_t *)Op, lse, redo, g, tok_delta);
}

}  // namespace pbs
