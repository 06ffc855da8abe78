// ssd_prefill on bf16 matrix cores: the Mamba-2 recurrence (paper Eqs. "ssm_state_update",
// "ssm_output") in its chunked form, i.e. the unrolled sum (Eq. "ssm_unrolled") split at
// 64-token boundaries, with the recurrent state of a head kept in the registers of the waves
// that own it for a whole segment of the sequence.
//
// Decomposition.  One workgroup owns 32*NC consecutive channels of one head (NC = 2: the whole
// head when P = 64) -- or, NH = 2, two whole heads of one group -- and one segment of the
// sequence, which it walks in 64-token steps.  Per step and head, with l_t the in-step cumulative
// sum of dt*A (log2 units):
//   (a) G^T[j,t] = b_j . c_t                                      contraction over the state dim n
//   (b) M[t,j]   = G^T[j,t] * 2^(l_t-l_j) * dt_j  for j <= t, else 0;  M[t,t] += D   (fp32, then bf16)
//   (c) Y^T[p,t] = sum_j x_j[p] M[t,j]                            contraction over tokens
//   (d) Y^T[p,t] += 2^(l_t) * sum_n S[p,n] c_t[n]                 S = state before the step
//   (e) S^T[n,p] = 2^(l_Q) S^T[n,p] + sum_j b_j[n] (w_j x_j[p]),  w_j = dt_j 2^(l_Q-l_j)
// every product a v_mfma_f32_16x16x32_bf16 (the skip term D x_t of the output rides on (c) through
// the diagonal of M).  (a) and (b) depend on the head only, not on the channel: two "G waves" per
// head do them once, two query blocks of 16 tokens each, keep the weights M in registers -- the
// accumulators of (a), rounded to bf16, are the B operand of (c) as they stand -- and go on to (c)
// for all the head's channels and to the outputs.  (d) and (e) belong to NC "compute waves" per
// head, one per slab of 32 channels, which hold their slab's state S^T[n, 32] in fp32 accumulator
// registers from the first step to the last.  The accumulator layout of (e) is at the same time
// the A-operand layout of (d) (the contraction index n runs over the accumulator rows a lane
// holds), so the state is converted to bf16 in registers and never passes through LDS; the
// carried part (d) of a step's outputs goes to the G waves through LDS in accumulator layout,
// rounded to bf16 (8 bytes per lane, no bank conflicts).
//
// Waves (NH (NC + 2) + 4): per head NC compute waves and 2 G waves; one wave each that only
// requests the asynchronous global -> LDS copies of the B tiles, the C tiles and the x tiles; a
// helper wave that requests dt three steps ahead and turns it into the scan l_t, the key factors
// of (b), the weights of (e) and the carries of (d) one step ahead (and keeps the row tables of
// the gather form).  One LDS-only barrier per step.  The outputs of a step leave one step late:
// the G waves keep (c) of step i in registers, the compute waves leave the carried part (d) of
// step i in LDS (bf16, double-buffered), the barrier that ends the step publishes it, and the G
// waves add the two and store them while the arithmetic of step i + 1 runs.
//
// One head per workgroup (NH = 1): 8 waves, two per SIMD, 256 registers each; tiles two steps
// ahead (rings of 3), every LDS read of a step requested at its start.  Two heads (NH = 2, P = 64
// and an even number of heads per group): 12 waves, three per SIMD -- a compute wave, a G wave
// and a copy wave -- so that the vector work of one arithmetic wave runs under the matrix
// products and LDS round trips of the other, and the B and C tiles cross the CU's copy path once
// for both heads.  That leaves 168 registers per wave and LDS for rings of 2 (tiles one step
// ahead): reads are requested where they are needed instead of at the start of the step.
//
// Segments.  A head is a serial chain over time; to fill the chip the sequence is cut into a few
// long segments that run side by side, each from a zero state (the first from S_in).  A segment
// leaves its final local state and its total decay in the workspace; a second, small kernel adds
// what the true incoming state contributes to the first tokens of each later segment,
//   y_t += 2^(l_t) * E c_t,   E = state at the segment's start, l_t = decay since then,
// for as many 64-token tiles as 2^(l_t) is not yet zero in fp32 (a handful at the decay rates of
// a trained layer, the whole segment if A = 0: always exact), and completes S_out.
//
// GATHER: token t of the sequence is row idx[t] (t < K) or N + t - K of the tensors, i.e. the
// kernel reads the uncompacted x, dt, B, C through the kept-index list instead of a compacted copy.
#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kQ = 64;       // tokens per step
constexpr int kRD = 4;       // dt rows in LDS (requested kRD - 1 steps ahead)
// per head NC compute waves + 2 G waves; 3 copy waves + helper per workgroup
constexpr int threads_for(int NC, int NH) { return 64 * (NH * (NC + 2) + 4); }
constexpr float kLog2e = 1.4426950408889634f;

struct SegArgs {
    const bf16_t *x;
    const float *dt, *A;
    const bf16_t *B, *C;
    const float *D, *S_in;
    bf16_t *y;
    float *S_out;  // final state [H, P, n] or null
    float *lend;   // [nseg - 1, H, P, n]: final local state of every segment but the last
    float *ltot;   // [nseg, H]: total log2 decay of every segment
    const int32_t *idx;
    int N, K, T, H, P, G;
    int nseg, seg_steps;  // segments and 64-token steps per segment (the last may be shorter)
    int wg_per_seg;       // H * P / (32 * NC)
};

template <int NS, int NC, int NH>
struct LdsS {
    static constexpr int kRB = NH == 1 ? 3 : 2;  // B / C tiles in LDS (requested kRB - 1 steps ahead)
    static constexpr int kRX = NH == 1 ? 3 : 2;  // x tiles in LDS
    // One B and one C tile, each filled by one wave.  Pitches by measurement (bytes per clock and CU of the
    // read patterns below in a loop of their own, row pitch in 4-byte words modulo the 64 banks):
    //   16-byte reads, lane = (row lane % 16, piece lane / 16):            8: 180    4: 117
    //   transposing reads, 8 consecutive rows per half wave:              8: 118    4: 108
    //   transposing reads, every other row (state_tok below):             8: 123    4: 130
    //   8-byte reads of 16 rows, one instruction each:                    8: 115    4: 144
    //   the same two at a time (ds_read2_b64, what the compiler makes):   8:  32    4:  64
    // B tile (16-byte row reads in (a), transposing reads in (e)): 2 pad vectors, pitch 72 = 8 mod 64.
    // C tile (16-byte row reads in (a), 8-byte row reads in (d), issued one by one): 1 pad vector, 68 = 4.
    using BT = AsyncTile<kQ, NS / 8, 1, 2, true>;
    using CT = AsyncTile<kQ, NS / 8, 1, 1, true>;
    using XT = AsyncTile<kQ, NH * NC * 4, 1, 1, true>;  // x tile of the workgroup's channels, 1 pad vector per row (2 changed nothing)
    static constexpr int kBP = BT::kPitch;         // bf16 elements per row of the B tiles
    static constexpr int kCP = CT::kPitch;         // ... of the C tiles
    static constexpr int kXP = XT::kPitch;         // ... of the x tiles
    struct alignas(16) TileBC {
        bf16_t c[CT::kBytes / 2];
        bf16_t b[BT::kBytes / 2];
    };
    struct alignas(16) TileX {
        bf16_t x[XT::kBytes / 2];
    };
    struct alignas(16) Scan {
        float ell[kQ];    // inclusive cumulative sum of dt*A*log2(e) inside the step
        float dtv[kQ];    // dt (0 past the end of the sequence)
        float fw[96];     // key factors of query block W = 1..3 at fw_at(W): dt_j * 2^(l_{16W-1} - l_j), j < 16W
        float w[kQ];      // weights of the state update: w_j = dt_j * 2^(l_Q - l_j)
        float carry[kQ];  // 2^(l_t); carry[kQ - 1] is the decay of the state over the step
    };
    static constexpr int fw_at(int W) { return W <= 1 ? 0 : W == 2 ? 16 : 48; }
    TileBC bc[kRB];
    TileX xr[kRX];
    float dt[NH][kRD][kQ];
    Scan scan[NH][2];
    bf16x4 yin[2][NH][8 * NC][64];  // carried part of the outputs of step i, [i % 2][head][query block * 2 NC + channel tile][lane]
    uint32_t rowtab[4][kQ];  // gather mode: source row of every token of local step i, i % 4 = slot
    int32_t rawidx[4][kQ];   // gather mode: entries of the kept-index list for local step i, i % 4 = slot
};

static_assert(sizeof(LdsS<128, 2, 1>) <= 160 * 1024 && sizeof(LdsS<128, 2, 2>) <= 160 * 1024, "one workgroup must fit the 160 KB of LDS of a CU");

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }
__device__ __forceinline__ float read_lane_f32(float v, int l) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
__device__ __forceinline__ bf16x8 cat8(bf16x4 lo, bf16x4 hi) {
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
__device__ __forceinline__ bf16x4 to_bf16x4(f32x4 v) {
    return bf16x4{(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
}

// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding
// (gfx9 layout: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14); n < 64.
constexpr int vm_wait_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// The k slots of a token-contracted fragment: slot s of lane group lb in token half kr is token
// 32 kr + 4 lb + (s & 3) + 16 (s >> 2).  Every operand that is contracted over tokens (x in (c)
// and (e), b in (e), M in (c), the weights w) uses this one order.

// The four token-contracted fragments of the x tile for a slab of 32 channels at column c0
// ([kr = token half][pt = channel half]).  Issued early (issue_x_frags), usable after take_x_frags.
// `row`: the row of a 16-token block whose 8-byte piece this lane passes (4 lb + lr / 4 for the order above).
template <int PITCH>
__device__ __forceinline__ void issue_x_frags(const bf16_t *xt, int c0, int row, int lr, strd_s16x4 (&r)[8]) {
    constexpr int R = PITCH * 2;  // row pitch in bytes
    lds_issue_tr8<0, 16 * R, 32, 16 * R + 32, 32 * R, 48 * R, 32 * R + 32, 48 * R + 32>(
        xt + row * PITCH + c0 + 4 * (lr & 3), r);
}
// The state update (e) contracts over the tokens of a step, in any order as long as b, x and the
// weights w agree on it.  Its k slot (lb, j) of a 16-token block is token 8 (lb & 1) + 2 j + (lb >> 1):
// the two lane groups of a half wave then pass the even (or the odd) rows of the block to a
// transposing read, 8 rows two apart, which at a row pitch of 4 (B tile) or 36 (x tile) words modulo 64
// start 8 banks apart -- no two of them share a bank.  ((c) keeps the order above: its weights come out
// of the accumulators of (a) in that order.)
__device__ __forceinline__ int state_tok(int lb, int j) { return 8 * (lb & 1) + 2 * j + (lb >> 1); }
__device__ __forceinline__ void take_x_frags(strd_s16x4 (&r)[8], bf16x8 (&xf)[2][2]) {
    lds_settle8(r);
    xf[0][0] = tr_pair(r[0], r[1]);
    xf[0][1] = tr_pair(r[2], r[3]);
    xf[1][0] = tr_pair(r[4], r[5]);
    xf[1][1] = tr_pair(r[6], r[7]);
}

// The 8-byte pieces of one c row that a lane needs as B operand of (d): elements 32 ks + 4 lb .. + 3 and
// the same 16 further on, for every k-step -- 2 KS plain reads 32 bytes apart, requested together and
// waited for separately (same contract as lds_issue_tr8 / lds_settle8).
template <int KS>
__device__ __forceinline__ void issue_c_pieces(const bf16_t *p, strd_s16x4 (&r)[2 * KS]) {
    static_assert(KS == 2 || KS == 4, "state sizes 64 and 128");
    const uint32_t a = lds_offset(p);
    if constexpr (KS == 4)
        asm volatile(
            "ds_read_b64 %0, %8\n\tds_read_b64 %1, %8 offset:32\n\tds_read_b64 %2, %8 offset:64\n\t"
            "ds_read_b64 %3, %8 offset:96\n\tds_read_b64 %4, %8 offset:128\n\tds_read_b64 %5, %8 offset:160\n\t"
            "ds_read_b64 %6, %8 offset:192\n\tds_read_b64 %7, %8 offset:224"
            : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7])
            : "v"(a)
            : "memory");
    else
        asm volatile(
            "ds_read_b64 %0, %4\n\tds_read_b64 %1, %4 offset:32\n\tds_read_b64 %2, %4 offset:64\n\t"
            "ds_read_b64 %3, %4 offset:96"
            : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
            : "v"(a)
            : "memory");
}
template <int KS>
__device__ __forceinline__ void settle_c_pieces(strd_s16x4 (&r)[2 * KS]) {
    if constexpr (KS == 4)
        lds_settle8(r);
    else
        lds_settle4(r);
}

// ---- compute wave: the slab of 32 channels at column 32 * cw of the workgroup's x tile: (d), (e) ----
template <int NS, int NC, int NH, bool GATHER>
__device__ __forceinline__ void compute_wave(LdsS<NS, NC, NH> &lds, const SegArgs &a, int hh, int cw, int h, int pin, int nloc,
                                             const float *s_src, float *s_dst) {
    using L = LdsS<NS, NC, NH>;
    constexpr int KS = NS / 32;  // k-steps of the products contracted over n
    constexpr int NT = NS / 16;  // 16-row tiles of the state
    const int lane = threadIdx.x & 63, lr = lane & 15, lb = lane >> 4;
    const int xcol = 32 * (NC * hh + cw);  // first column of the slab in the x tile
    const int scol = 32 * cw;              // ... in the head

    // state: S^T[n][p] tiles, rows n = 16 nt + 4 lb + i, columns p = pin + 32 cw + 16 pt + lr
    f32x4 sacc[NT][2];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int pt = 0; pt < 2; ++pt) {
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (s_src) v = *reinterpret_cast<const f32x4 *>(s_src + ((size_t)h * a.P + pin + scol + 16 * pt + lr) * NS + 16 * nt + 4 * lb);
            sacc[nt][pt] = v;
        }

    if (GATHER) __syncthreads();  // prologue barriers: (row tables written |)
    __syncthreads();              // first copies landed |
    __syncthreads();              // scan of the first step

    for (int i = 0; i < nloc; ++i) {
        const typename L::Scan &sc = lds.scan[hh][i & 1];
        const typename L::TileBC &tb = lds.bc[i % L::kRB];
        const bf16_t *xt = lds.xr[i % L::kRX].x;
        // ---- LDS reads that do not depend on the arithmetic of the step are requested first: x fragments
        // and the first b^T fragments (transposing reads, for (e)), the weights.  With three waves on a SIMD
        // (NH = 2) the registers do not allow that, and the other waves cover the round trip: there these
        // reads are requested after (d).
        constexpr int R = L::kBP * 2;
        constexpr bool kEarly = NH == 1;
        strd_s16x4 xr8[8], ba[8], bb[8];
        const int trow = state_tok(lb, lr >> 2);  // the row of a 16-token block this lane passes to a transposing read
        const bf16_t *bbase = &tb.b[trow * L::kBP + 4 * (lr & 3)];
        f32x4 wv[2][2];
        auto request_e = [&]() __attribute__((always_inline)) {
            issue_x_frags<L::kXP>(xt, xcol, trow, lr, xr8);
            // state tile d of a group of four: columns + 16 d of the b tile; rows + 0, 16 (token half 0: slots
            // 0-3, 4-7), + 32, 48 (token half 1); ba: tiles 0, 1; bb: tiles 2, 3
            lds_issue_tr8<0, 16 * R, 32 * R, 48 * R, 32, 16 * R + 32, 32 * R + 32, 48 * R + 32>(bbase, ba);
            lds_issue_tr8<64, 16 * R + 64, 32 * R + 64, 48 * R + 64, 96, 16 * R + 96, 32 * R + 96, 48 * R + 96>(bbase, bb);
#pragma unroll
            for (int kr = 0; kr < 2; ++kr)
#pragma unroll
                for (int hi = 0; hi < 2; ++hi)
#pragma unroll
                    for (int e = 0; e < 4; ++e) wv[kr][hi][e] = sc.w[32 * kr + 16 * hi + state_tok(lb, e)];
        };
        if constexpr (kEarly) request_e();
        const float dq = sc.carry[kQ - 1];
        // (d): Y^T[p, t] = sum_n S[p, n] c_t[n] (the factor 2^(l_t) is applied where the outputs are summed).
        // A operand straight from the accumulators: the lane holds rows 4 lb .. 4 lb + 3 of state tiles
        // 2 ks and 2 ks + 1 for column p = lr, i.e. the k slots n = 32 ks + 4 lb + s (s < 4),
        // 32 ks + 16 + 4 lb + s - 4 (s >= 4) of row p; the c fragments are read in the same slot order
        // (two 8-byte reads).  Once the bf16 copy exists the accumulators are free: their decay, which
        // (e) needs, is interleaved with the products of (d), so that vector and matrix pipe overlap.
        bf16x8 sb[2][KS];
#pragma unroll
        for (int pt = 0; pt < 2; ++pt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) sb[pt][ks] = cat8(to_bf16x4(sacc[2 * ks][pt]), to_bf16x4(sacc[2 * ks + 1][pt]));
        // (the 8-byte pieces are read by instructions of their own, a query block ahead: paired into
        // ds_read2_b64, as the compiler does with ordinary loads, they run at less than half the rate)
        strd_s16x4 cr[2][2 * KS];
        const bf16_t *cbase = &tb.c[lr * L::kCP + 4 * lb];
        issue_c_pieces<KS>(cbase, cr[0]);
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            bf16x8 cf[KS];
            settle_c_pieces<KS>(cr[tt & 1]);
            if (tt < 3) issue_c_pieces<KS>(cbase + 16 * (tt + 1) * L::kCP, cr[(tt + 1) & 1]);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) cf[ks] = tr_pair(cr[tt & 1][2 * ks], cr[tt & 1][2 * ks + 1]);
#pragma unroll
            for (int pt = 0; pt < 2; ++pt) {
                f32x4 yin = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) yin = mfma16(sb[pt][ks], cf[ks], yin);
                lds.yin[i & 1][hh][tt * (2 * NC) + 2 * cw + pt][lane] = to_bf16x4(yin);  // to the G wave of query block tt
            }
            // a quarter of the state's decay per query block
#pragma unroll
            for (int nt = tt * (NT / 4); nt < (tt + 1) * (NT / 4); ++nt)
#pragma unroll
                for (int pt = 0; pt < 2; ++pt) sacc[nt][pt] *= dq;
        }
        // (e): S^T = 2^(l_Q) S^T + b^T (w x).  The x fragments, weighted in registers, are the B operand.
        if constexpr (!kEarly) request_e();
        bf16x8 xf[2][2], xwf[2][2];
        take_x_frags(xr8, xf);  // waits for every read requested above
#pragma unroll
        for (int kr = 0; kr < 2; ++kr)
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int e = 0; e < 8; ++e) xwf[kr][pt][e] = (bf16_t)((float)xf[kr][pt][e] * wv[kr][e >> 2][e & 3]);
#pragma unroll
        for (int n4 = 0; n4 < NT; n4 += 4) {
            lds_settle8(ba);
            lds_settle8(bb);
            bf16x8 bt[4][2];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const strd_s16x4 *r = d < 2 ? &ba[4 * d] : &bb[4 * (d - 2)];
                bt[d][0] = tr_pair(r[0], r[1]);
                bt[d][1] = tr_pair(r[2], r[3]);
            }
            if (n4 + 4 < NT) {  // next group of four tiles: columns + 64
                lds_issue_tr8<128, 16 * R + 128, 32 * R + 128, 48 * R + 128, 160, 16 * R + 160, 32 * R + 160, 48 * R + 160>(bbase, ba);
                lds_issue_tr8<192, 16 * R + 192, 32 * R + 192, 48 * R + 192, 224, 16 * R + 224, 32 * R + 224, 48 * R + 224>(bbase, bb);
            }
            // independent products back to back: first token half of all eight tiles, then the second
#pragma unroll
            for (int kr = 0; kr < 2; ++kr)
#pragma unroll
                for (int d = 0; d < 4; ++d)
#pragma unroll
                    for (int pt = 0; pt < 2; ++pt) sacc[n4 + d][pt] = mfma16(bt[d][kr], xwf[kr][pt], sacc[n4 + d][pt]);
        }
        lds_barrier();  // the step is over
    }

    if (s_dst) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
                *reinterpret_cast<f32x4 *>(s_dst + ((size_t)h * a.P + pin + scol + 16 * pt + lr) * NS + 16 * nt + 4 * lb) =
                    sacc[nt][pt];
    }
}

// ---- G wave GW: (a), (b), (c) and the outputs of the query blocks {0, 3} (GW = 0) or {1, 2} (GW = 1) ----
// The outputs of a step leave one step late: (a)-(c) of step i are summed up in registers during step i,
// the carried part arrives from the compute waves with the barrier that ends the step.
template <int NS, int NC, int NH, int GW, bool GATHER>
__device__ __forceinline__ void g_wave(LdsS<NS, NC, NH> &lds, const SegArgs &a, int hh, int h, int chan0, int tok0, int nloc) {
    using L = LdsS<NS, NC, NH>;
    const int xc0 = 32 * NC * hh;  // first column of the head in the x tile
    // Sharing a SIMD with a compute wave, the G waves are the last to reach the barrier of a step (by about a
    // tenth of the step): their instructions go first (-1.5 % kernel time).
    if (NH == 2) __builtin_amdgcn_s_setprio(2);
    constexpr int KS = NS / 32;
    constexpr int PT = 2 * NC;                                  // 16-channel tiles of the workgroup
    constexpr int TA = GW == 0 ? 0 : 1, TB = GW == 0 ? 3 : 2;  // the two query blocks of this wave
    const int lane = threadIdx.x & 63, lr = lane & 15, lb = lane >> 4;
    const int HP = a.H * a.P;
    // The skip term D x_t rides on (c): D is added to the diagonal of the weights, M[t, t] += D, so that
    // X M carries it (rounded to bf16 with the weight, like every other term of the sum).
    const float Dh = a.D ? a.D[h] : 0.f;
    f32x4 dskip;
#pragma unroll
    for (int e = 0; e < 4; ++e) dskip[e] = 4 * lb + e == lr ? Dh : 0.f;
    f32x4 ya[PT], yb[PT];  // (c) of the step before, until its carried part arrives
    // Outputs of a step: what is in ya / yb plus the carried part the compute waves left in LDS.
    // A lane holds 4 channels of one token, i.e. 8 bytes of a 32 PT-byte row of y; stored like that,
    // every store instruction would touch 16 rows with 32 bytes each.  The rows are turned in LDS first
    // -- in the slots of the carried parts this wave has just read, which nobody needs before the step
    // after next -- so that a lane stores 16 bytes and a store instruction writes whole rows.  The three
    // stages (read the carried part; add and write the rows; read them back and store) are spread over
    // the arithmetic of the next step, so that their LDS round trips are not waited for.
    constexpr int NCH = 2 * PT;    // 16-byte pieces per row of the workgroup's channels
    constexpr int RPI = 64 / NCH;  // rows per store instruction
    const int srow = lane / NCH, spc = lane % NCH;
    bf16x4 ia[PT], ib[PT];
    bf16x8 va[16 / RPI], vb[16 / RPI];
    float cra = 0.f, crb = 0.f;  // 2^(l_t) of this lane's tokens in the step whose outputs are waiting
    auto emit_read = [&](int j) __attribute__((always_inline)) {
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            ia[pt] = lds.yin[j & 1][hh][TA * PT + pt][lane];
            ib[pt] = lds.yin[j & 1][hh][TB * PT + pt][lane];
        }
    };
    auto emit_turn = [&](int j) __attribute__((always_inline)) {
        char *sta = reinterpret_cast<char *>(&lds.yin[j & 1][hh][TA * PT][0]), *stb = reinterpret_cast<char *>(&lds.yin[j & 1][hh][TB * PT][0]);
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            bf16x4 oa, ob;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                oa[e] = (bf16_t)(ya[pt][e] + cra * (float)ia[pt][e]);
                ob[e] = (bf16_t)(yb[pt][e] + crb * (float)ib[pt][e]);
            }
            // row lr, piece 2 pt + lb / 2 (pieces swizzled by the row so that rows do not share banks), half lb % 2
            const int off = lr * (16 * NCH) + (((2 * pt + (lb >> 1)) ^ (lr & (NCH - 1))) << 4) + ((lb & 1) << 3);
            *reinterpret_cast<bf16x4 *>(sta + off) = oa;
            *reinterpret_cast<bf16x4 *>(stb + off) = ob;
        }
    };
    auto emit_back = [&](int j) __attribute__((always_inline)) {
        const char *sta = reinterpret_cast<const char *>(&lds.yin[j & 1][hh][TA * PT][0]), *stb = reinterpret_cast<const char *>(&lds.yin[j & 1][hh][TB * PT][0]);
#pragma unroll
        for (int k = 0; k < 16 / RPI; ++k) {
            const int r = srow + RPI * k;
            const int off = r * (16 * NCH) + ((spc ^ (r & (NCH - 1))) << 4);
            va[k] = *reinterpret_cast<const bf16x8 *>(sta + off);
            vb[k] = *reinterpret_cast<const bf16x8 *>(stb + off);
        }
    };
    auto emit_store = [&](int j) __attribute__((always_inline)) {
        const int tbase = tok0 + j * kQ;
#pragma unroll
        for (int k = 0; k < 16 / RPI; ++k) {
            const int r = srow + RPI * k;
            if (tbase + 16 * TA + r < a.T)
                *reinterpret_cast<bf16x8 *>(a.y + (size_t)(tbase + 16 * TA + r) * HP + chan0 + 8 * spc) = va[k];
            if (tbase + 16 * TB + r < a.T)
                *reinterpret_cast<bf16x8 *>(a.y + (size_t)(tbase + 16 * TB + r) * HP + chan0 + 8 * spc) = vb[k];
        }
    };
    if (GATHER) __syncthreads();
    __syncthreads();
    __syncthreads();

    for (int i = 0; i < nloc; ++i) {
        const typename L::Scan &sc = lds.scan[hh][i & 1];
        const typename L::TileBC &tb = lds.bc[i % L::kRB];
        const bf16_t *xt = lds.xr[i % L::kRX].x;
        const bool prev = i > 0;  // uniform: the step before has outputs waiting
        // fragments: b rows of key blocks 0..TB, c rows of the two query blocks
        strd_s16x4 xr8[NC][8];
        f32x4 ga[TA + 1], gb[TB + 1];
#pragma unroll
        for (int jt = 0; jt <= TA; ++jt) ga[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int jt = 0; jt <= TB; ++jt) gb[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto frag_b = [&](int jt, int ks) __attribute__((always_inline)) {
            return *reinterpret_cast<const bf16x8 *>(&tb.b[(16 * jt + lr) * L::kBP + 32 * ks + 8 * lb]);
        };
        auto frag_c = [&](int tt, int ks) __attribute__((always_inline)) {
            return *reinterpret_cast<const bf16x8 *>(&tb.c[(16 * tt + lr) * L::kCP + 32 * ks + 8 * lb]);
        };
        if constexpr (NH == 1) {
            // all fragments requested before (a)
            bf16x8 bf[TB + 1][KS], cfa[KS], cfb[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int jt = 0; jt <= TB; ++jt) bf[jt][ks] = frag_b(jt, ks);
                cfa[ks] = frag_c(TA, ks);
                cfb[ks] = frag_c(TB, ks);
            }
            __builtin_amdgcn_sched_barrier(0);
            // (a)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int jt = 0; jt <= TA; ++jt) ga[jt] = mfma16(bf[jt][ks], cfa[ks], ga[jt]);
#pragma unroll
                for (int jt = 0; jt <= TB; ++jt) gb[jt] = mfma16(bf[jt][ks], cfb[ks], gb[jt]);
            }
        } else {
            // three waves share the SIMD's registers: the fragments of one k-step ahead of the products only
            bf16x8 bf[2][TB + 1], cfa[2], cfb[2];
            auto request_a = [&](int ks) __attribute__((always_inline)) {
#pragma unroll
                for (int jt = 0; jt <= TB; ++jt) bf[ks & 1][jt] = frag_b(jt, ks);
                cfa[ks & 1] = frag_c(TA, ks);
                cfb[ks & 1] = frag_c(TB, ks);
            };
            request_a(0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks + 1 < KS) request_a(ks + 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int jt = 0; jt <= TA; ++jt) ga[jt] = mfma16(bf[ks & 1][jt], cfa[ks & 1], ga[jt]);
#pragma unroll
                for (int jt = 0; jt <= TB; ++jt) gb[jt] = mfma16(bf[ks & 1][jt], cfb[ks & 1], gb[jt]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // while (a) runs: the x fragments of every channel tile (for (c)) and the carried part of the step
        // before (published by the barrier that ended it) are requested
        // (NH = 2: after (b) -- three waves share the SIMD's registers, and cover the round trip)
        __builtin_amdgcn_sched_barrier(0);
        auto request_c = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int c = 0; c < NC; ++c) issue_x_frags<L::kXP>(xt, xc0 + 32 * c, 4 * lb + (lr >> 2), lr, xr8[c]);
            if (prev) emit_read(i - 1);
        };
        if constexpr (NH == 1) request_c();
        // what (b) needs from the scan of the head
        const float el_a = sc.ell[16 * TA + lr], el_b = sc.ell[16 * TB + lr];
        const float ref_a = TA > 0 ? sc.ell[16 * TA - 1] : 0.f, ref_b = sc.ell[16 * TB - 1];
        const f32x4 elj_a = *reinterpret_cast<const f32x4 *>(&sc.ell[16 * TA + 4 * lb]);
        const f32x4 elj_b = *reinterpret_cast<const f32x4 *>(&sc.ell[16 * TB + 4 * lb]);
        const f32x4 dtj_a = *reinterpret_cast<const f32x4 *>(&sc.dtv[16 * TA + 4 * lb]);
        const f32x4 dtj_b = *reinterpret_cast<const f32x4 *>(&sc.dtv[16 * TB + 4 * lb]);
        f32x4 fja[TA > 0 ? TA : 1] = {}, fjb[TB];
#pragma unroll
        for (int jt = 0; jt < TA; ++jt) fja[jt] = *reinterpret_cast<const f32x4 *>(&sc.fw[L::fw_at(TA) + 16 * jt + 4 * lb]);
#pragma unroll
        for (int jt = 0; jt < TB; ++jt) fjb[jt] = *reinterpret_cast<const f32x4 *>(&sc.fw[L::fw_at(TB) + 16 * jt + 4 * lb]);
        __builtin_amdgcn_sched_barrier(0);
        // (b): blocks below the diagonal: 2^(l_t - l_j) dt_j = 2^(l_t - l_ref) * fw[j] with l_ref the scan at
        // the last token before the query block (both exponents <= 0); diagonal block: direct, masked.
        // The weights, rounded to bf16, are the B operand of (c) as they stand in the registers.
        auto weigh = [&](int tt, int jt, f32x4 g, float el_t, float e_ref, f32x4 fj, f32x4 elj, f32x4 dtj)
                         __attribute__((always_inline)) -> bf16x4 {
            bf16x4 mv;
            if (jt < tt) {
#pragma unroll
                for (int e = 0; e < 4; ++e) mv[e] = (bf16_t)(g[e] * e_ref * fj[e]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float val = g[e] * fast_exp2(el_t - elj[e]) * dtj[e] + dskip[e];
                    mv[e] = (bf16_t)((4 * lb + e <= lr) ? val : 0.f);  // causal mask
                }
            }
            return mv;
        };
        const float era = TA > 0 ? fast_exp2(el_a - ref_a) : 0.f, erb = fast_exp2(el_b - ref_b);
        bf16x4 ma[4], mb[4];
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            ma[jt] = mb[jt] = bf16x4{(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
            if (jt <= TA) ma[jt] = weigh(TA, jt, ga[jt <= TA ? jt : 0], el_a, era, fja[jt < TA ? jt : 0], elj_a, dtj_a);
            if (jt <= TB) mb[jt] = weigh(TB, jt, gb[jt <= TB ? jt : 0], el_b, erb, fjb[jt < TB ? jt : 0], elj_b, dtj_b);
        }
        // the rows of the step before are summed, written for turning and read back; they travel under (c)
        if constexpr (NH != 1) {
            __builtin_amdgcn_sched_barrier(0);
            request_c();
        }
        if (prev) {
            emit_turn(i - 1);
            emit_back(i - 1);
        }
        // (c): Y^T[p, t] = sum_j x_j[p] M[t, j]; query block tt needs the key halves kr <= tt / 2
        bf16x8 xf[NC][2][2];
#pragma unroll
        for (int c = 0; c < NC; ++c) take_x_frags(xr8[c], xf[c]);
        // the stores of the step before go out now, not at the end of the step: the copies of the step
        // share the CU's path to memory with them and were requested at its start
        if (prev) emit_store(i - 1);
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            ya[pt] = yb[pt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kr = 0; kr < 2; ++kr) {
                if (2 * kr <= TA) ya[pt] = mfma16(xf[pt >> 1][kr][pt & 1], cat8(ma[2 * kr], ma[2 * kr + 1]), ya[pt]);
                if (2 * kr <= TB) yb[pt] = mfma16(xf[pt >> 1][kr][pt & 1], cat8(mb[2 * kr], mb[2 * kr + 1]), yb[pt]);
            }
        }
        cra = sc.carry[16 * TA + lr];
        crb = sc.carry[16 * TB + lr];
        lds_barrier();  // the step is over
    }
    emit_read(nloc - 1);
    emit_turn(nloc - 1);
    emit_back(nloc - 1);
    emit_store(nloc - 1);
}

// Source row of token t of the sequence (gather form); an index outside [0, N) is clamped into
// the tensors instead of faulting.
__device__ __forceinline__ uint32_t gather_row(const SegArgs &a, int t, int32_t kept) {
    const uint32_t last_row = (uint32_t)(a.N + (a.T - a.K) - 1);
    return min((uint32_t)(t < a.K ? kept : a.N + (t - a.K)), last_row);
}

// ---- helper wave: dt copies, the scans of the workgroup's heads, the row tables of the gather form ----
template <int NS, int NC, int NH, bool GATHER>
__device__ __forceinline__ void helper_wave(LdsS<NS, NC, NH> &lds, const SegArgs &a, int h0, int tok0, int nloc, int seg) {
    using L = LdsS<NS, NC, NH>;
    const int lane = threadIdx.x & 63;
    float Al2[NH];
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) Al2[hh] = a.A[h0 + hh] * kLog2e;
    __builtin_amdgcn_s_setprio(3);
    auto token_of = [&](int i) { return min(tok0 + i * kQ + lane, a.T - 1); };
    auto kept_of = [&](int i) -> int32_t { return a.idx[min(token_of(i), a.K - 1)]; };  // K >= 1 in gather mode
    auto request_kept = [&](int i) __attribute__((always_inline)) {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(a.idx + min(token_of(i), a.K - 1)),
                                         (__attribute__((address_space(3))) void *)lds.rawidx[i & 3], 4, 0, 0);
    };
    const uint32_t dt_row = (uint32_t)a.H * 4;
    auto request_dt = [&](int i) __attribute__((always_inline)) {  // 64 lanes x 4 bytes per head; rows past T re-read the last row
        const uint32_t row = GATHER ? lds.rowtab[i & 3][lane] : (uint32_t)token_of(i);
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(reinterpret_cast<const char *>(a.dt) + row * dt_row + (uint32_t)(h0 + hh) * 4),
                (__attribute__((address_space(3))) void *)lds.dt[hh][i % kRD], 4, 0, 0);
    };
    // scan of dt*A of local step i of head hh, the key factors of (b), the weights of (e), the carries
    // of (d); returns the total log2 decay of the step
    auto make_scan = [&](int hh, int i, float raw) __attribute__((always_inline)) -> float {
        const float dv = (tok0 + i * kQ + lane < a.T) ? raw : 0.f;
        const float inc = wave_inclusive_scan_f32(dv * Al2[hh]);
        typename L::Scan &m = lds.scan[hh][i & 1];
        const float tot = read_lane_f32(inc, kQ - 1);
        m.ell[lane] = inc;
        m.dtv[lane] = dv;
        m.w[lane] = dv * fast_exp2(tot - inc);
        m.carry[lane] = fast_exp2(inc);
#pragma unroll
        for (int wq = 1; wq < 4; ++wq) {  // only tokens j < 16 * wq are read; the exponent is <= 0 for them
            const float lref = read_lane_f32(inc, 16 * wq - 1);
            if (lane < 16 * wq) m.fw[L::fw_at(wq) + lane] = dv * fast_exp2(lref - inc);
        }
        return tot;
    };
    constexpr int kNewest = NH + (GATHER ? 1 : 0);  // copies requested per step

    if (GATHER) {
#pragma unroll
        for (int i = 0; i < 4; ++i) lds.rowtab[i][lane] = gather_row(a, token_of(i), kept_of(i));
        lds.rawidx[4 & 3][lane] = kept_of(4);  // read in steps 0 and 1, before the first copied entries
        lds.rawidx[5 & 3][lane] = kept_of(5);
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 3; ++i)
        if (i < nloc) request_dt(i);
    async_tile_wait();
    __syncthreads();  // first copies landed
    float ltot[NH];
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) ltot[hh] = make_scan(hh, 0, lds.dt[hh][0][lane]);
    __syncthreads();  // scan of the first step

    for (int i = 0; i < nloc; ++i) {
        // dt of step i + 1 landed before the barrier that ended the previous step (or in the prologue)
        float raw[NH];
#pragma unroll
        for (int hh = 0; hh < NH; ++hh) raw[hh] = lds.dt[hh][(i + 1) % kRD][lane];
        int32_t kept = 0;
        if (GATHER) kept = lds.rawidx[(i + 4) & 3][lane];
        __builtin_amdgcn_sched_barrier(0);
        const bool more = i + 3 < nloc;  // uniform; nothing past the segment is requested
        if (more) {
            request_dt(i + 3);                     // slot last read in step i - 2
            if (GATHER) request_kept(i + 6);       // slot last read in step i - 2
        }
        if (i + 1 < nloc) {                        // buffers last read in step i - 1
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) ltot[hh] += make_scan(hh, i + 1, raw[hh]);
        }
        if (GATHER) lds.rowtab[(i + 4) & 3][lane] = gather_row(a, token_of(i + 4), kept);  // slot last used in step i - 2
        if (more)
            __builtin_amdgcn_s_waitcnt(vm_wait_imm(kNewest));  // everything requested in earlier steps has landed
        else
            async_tile_wait();
        lds_barrier();
    }
    if (lane == 0 && a.ltot) {
#pragma unroll
        for (int hh = 0; hh < NH; ++hh) a.ltot[(size_t)seg * a.H + h0 + hh] = ltot[hh];
    }
}

// ---- copy waves: one tile stream each (WHAT = 0: x, 1: B, 2: C), as far ahead as the ring allows
// (two steps with three tiles, one step with two).  A wave that requests a copy stands still until
// the CU's copy path takes it, so these waves do nothing else.
template <int NS, int NC, int NH, int WHAT, bool GATHER>
__device__ __forceinline__ void copy_wave(LdsS<NS, NC, NH> &lds, const SegArgs &a, int col_bytes, int tok0, int nloc) {
    using L = LdsS<NS, NC, NH>;
    using TT = typename std::conditional<WHAT == 0, typename L::XT, typename std::conditional<WHAT == 1, typename L::BT, typename L::CT>::type>::type;
    constexpr int RING = WHAT == 0 ? L::kRX : L::kRB;
    const int lane = threadIdx.x & 63;
    __builtin_amdgcn_s_setprio(3);
    const char *src = reinterpret_cast<const char *>(WHAT == 0 ? a.x : WHAT == 1 ? a.B : a.C);
    const uint32_t row_bytes = WHAT == 0 ? (uint32_t)a.H * a.P * 2 : (uint32_t)a.G * NS * 2;
    int row_of[TT::kIssues];
    uint32_t col_of[TT::kIssues];
#pragma unroll
    for (int k = 0; k < TT::kIssues; ++k) {
        int cv;
        TT::slot(0, lane, k, row_of[k], cv);
        col_of[k] = (uint32_t)col_bytes + (uint32_t)cv * 16;
    }
    // dense form: this lane's byte offsets inside the 64 rows of a step, worked out once -- a step's requests
    // are then its first row (a uniform pointer) plus these, and cost the SIMD no vector instruction
    uint32_t voff[TT::kIssues];
#pragma unroll
    for (int k = 0; k < TT::kIssues; ++k) voff[k] = (uint32_t)row_of[k] * row_bytes + col_of[k];
    auto request = [&](int i) __attribute__((always_inline)) {
        bf16_t *dst = WHAT == 0 ? lds.xr[i % L::kRX].x : WHAT == 1 ? lds.bc[i % L::kRB].b : lds.bc[i % L::kRB].c;
        const int t0 = tok0 + i * kQ;
        if (!GATHER && t0 + kQ <= a.T) {  // uniform: every row of the step exists
            const char *base = src + (size_t)t0 * row_bytes;
#pragma unroll
            for (int k = 0; k < TT::kIssues; ++k) TT::issue(base + voff[k], dst, 0, k);
            return;
        }
#pragma unroll
        for (int k = 0; k < TT::kIssues; ++k) {
            const uint32_t row = GATHER ? lds.rowtab[i & 3][row_of[k]] : (uint32_t)min(t0 + row_of[k], a.T - 1);
            TT::issue(src + (size_t)row * row_bytes + col_of[k], dst, 0, k);
        }
    };
    static_assert((RING - 2) * TT::kIssues < 64, "vmcnt has 6 bits");

    if (GATHER) __syncthreads();  // row tables of steps 0..3 written
#pragma unroll
    for (int i = 0; i < RING - 1; ++i)
        if (i < nloc) request(i);
    async_tile_wait();
    __syncthreads();  // first copies landed
    __syncthreads();

    for (int i = 0; i < nloc; ++i) {
        const bool more = i + RING - 1 < nloc;  // uniform
        if (more) request(i + RING - 1);        // slot last read in step i - 1
        if (more && RING > 2)
            __builtin_amdgcn_s_waitcnt(vm_wait_imm((RING - 2) * TT::kIssues));  // the tile of step i + 1 has landed
        else
            async_tile_wait();
        lds_barrier();  // publishes it; with a ring of three this step's copies stay in flight
    }
}

template <int NS, int NC, int NH, bool GATHER>
__global__ __launch_bounds__(threads_for(NC, NH)) void ssd_seg_kernel(SegArgs a, int nunits) {
    using L = LdsS<NS, NC, NH>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    L &lds = *reinterpret_cast<L *>(smem_raw);

    const int unit = xcd_swizzle(blockIdx.x, nunits);
    if (unit >= nunits) return;
    const int seg = unit / a.wg_per_seg, u = unit % a.wg_per_seg;
    const int chan0 = u * (32 * NC * NH);  // NH = 2: two whole heads of one group (P = 32 NC)
    const int h0 = chan0 / a.P, pin = chan0 % a.P, g = h0 / (a.H / a.G);
    const int nsteps = (a.T + kQ - 1) / kQ;
    const int s0 = seg * a.seg_steps;
    const int nloc = min(a.seg_steps, nsteps - s0);
    const int tok0 = s0 * kQ;
    // where the segment's state comes from and goes to
    const float *s_src = seg == 0 ? a.S_in : nullptr;
    float *s_dst = seg == a.nseg - 1 ? a.S_out : a.lend + (size_t)seg * a.H * a.P * NS;
    // Wave i runs on SIMD i % 4.  NH = 1, NC = 2: the compute waves have SIMDs 0 and 1, the G waves 2 and 3, each
    // with one copy wave beside it.  NH = 2: every SIMD has one compute wave, one G wave and one copy wave, so
    // the vector work of one overlaps the matrix products of the other.
    const int wave = threadIdx.x >> 6;
    if (wave < NH * NC) {
        const int hh = NH == 1 ? 0 : wave / NC, cw = NH == 1 ? wave : wave % NC;
        compute_wave<NS, NC, NH, GATHER>(lds, a, hh, cw, h0 + hh, pin, nloc, s_src, s_dst);
        return;
    }
    const int r = wave - NH * NC;
    if (r < 2 * NH) {
        const int hh = NH == 1 ? 0 : r >> 1;
        if (r & 1)
            g_wave<NS, NC, NH, 1, GATHER>(lds, a, hh, h0 + hh, chan0 + hh * 32 * NC, tok0, nloc);
        else
            g_wave<NS, NC, NH, 0, GATHER>(lds, a, hh, h0 + hh, chan0 + hh * 32 * NC, tok0, nloc);
        return;
    }
    switch (r - 2 * NH) {
        case 0: copy_wave<NS, NC, NH, 1, GATHER>(lds, a, g * NS * 2, tok0, nloc); break;
        case 1: copy_wave<NS, NC, NH, 2, GATHER>(lds, a, g * NS * 2, tok0, nloc); break;
        case 2: helper_wave<NS, NC, NH, GATHER>(lds, a, h0, tok0, nloc, seg); break;
        default: copy_wave<NS, NC, NH, 0, GATHER>(lds, a, chan0 * 2, tok0, nloc); break;
    }
}

// ---- the contribution of the incoming state to the first tokens of segments 1.. and S_out -----
// grid = (boundary b = 1..nseg, head, z); b < nseg: y of segment b; b == nseg: S_out.
constexpr int kFixThreads = 256;
constexpr int kFixZ = 4;  // workgroups that share the tiles of one (segment, head)

template <int NS, bool GATHER>
__global__ __launch_bounds__(kFixThreads) void ssd_fix_kernel(SegArgs a) {
    constexpr int KS = NS / 32;
    const int b = 1 + blockIdx.x, h = blockIdx.y, z = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lr = lane & 15, lb = lane >> 4;
    const size_t seg_elems = (size_t)a.H * a.P * NS;
    // weight of segment s' < b in the state at the start of segment b: prod_{s' < u < b} 2^(ltot[u])
    // (uniform; the loops below stop at the first segment whose weight is zero)
    if (b == a.nseg) {
        if (!a.S_out) return;
        float f = fast_exp2(a.ltot[(size_t)(b - 1) * a.H + h]);
        const int per = a.P * NS / 4;  // float4s of the head's state
        for (int s = b - 2; s >= 0 && f != 0.f; --s) {
            const float *src = a.lend + (size_t)s * seg_elems + (size_t)h * a.P * NS;
            float *dst = a.S_out + (size_t)h * a.P * NS;
            for (int e = z * kFixThreads + threadIdx.x; e < per; e += kFixZ * kFixThreads) {
                f32x4 v = reinterpret_cast<const f32x4 *>(src)[e], o = reinterpret_cast<f32x4 *>(dst)[e];
                reinterpret_cast<f32x4 *>(dst)[e] = o + f * v;
            }
            f *= fast_exp2(a.ltot[(size_t)s * a.H + h]);
        }
        return;
    }
    const int HP = a.H * a.P, g = h / (a.H / a.G);
    const int tok0 = b * a.seg_steps * kQ;
    const int tend = min(a.T, (b + 1) * a.seg_steps * kQ);
    const float Al2 = a.A[h] * kLog2e;
    auto row_of = [&](int t) -> size_t {
        t = min(t, a.T - 1);
        return GATHER ? (size_t)gather_row(a, t, a.idx[min(t, a.K - 1)]) : (size_t)t;
    };
    // E = state at the start of segment b, as A-operand fragments (rows p = 16 pt + lr, k slots
    // n = 32 ks + 8 lb + s) of this wave's channel tiles pt = wave, wave + 4, ...; requested before it is
    // known whether any token needs it, so that its latency runs under that of the dt loads
    constexpr int kMaxPT = 1;  // channel tiles per wave held in registers (P <= 64); more are loaded when their turn comes
    const int npt = (a.P / 16 - wave + 3) / 4;
    bf16x8 ef[kMaxPT][KS];
    auto load_e = [&](int pt, bf16x8 (&out)[KS]) __attribute__((always_inline)) {
        f32x4 acc[KS][2];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc[ks][0] = acc[ks][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        float f = 1.f;
        for (int s = b - 1; s >= 0 && f != 0.f; --s) {
            const float *src = a.lend + (size_t)s * seg_elems + ((size_t)h * a.P + 16 * pt + lr) * NS + 8 * lb;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                acc[ks][0] += f * *reinterpret_cast<const f32x4 *>(src + 32 * ks);
                acc[ks][1] += f * *reinterpret_cast<const f32x4 *>(src + 32 * ks + 4);
            }
            f *= fast_exp2(a.ltot[(size_t)s * a.H + h]);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) out[ks] = cat8(to_bf16x4(acc[ks][0]), to_bf16x4(acc[ks][1]));
    };
    // dt of kFixZ tiles at once (lane = token); the first batch travels together with the E fragments
    float dv[kFixZ];
    auto load_dt = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < kFixZ; ++q) {
            const int t = tok0 + (k0 + q) * kQ + lane;
            dv[q] = t < tend ? a.dt[row_of(t) * a.H + h] : 0.f;
        }
    };
    load_dt(0);
    // (the workgroups of the first two tiles only: at the decay rates of a trained layer the later tiles of a
    // batch are rarely reached, and every workgroup that loads E reads 32 KB -- they fetch it when they need it)
    bool have_e = z < 2;  // uniform
    if (have_e) {
#pragma unroll
        for (int q = 0; q < kMaxPT; ++q)
            if (q < npt) load_e(wave + 4 * q, ef[q]);
    }
    float prefix = 0.f;  // log2 decay from the segment's start to the tile's start
    for (int k0 = 0; tok0 + k0 * kQ < tend; k0 += kFixZ) {
        if (k0 > 0) load_dt(k0);
        float cr = 0.f;
        bool dead = false;
#pragma unroll
        for (int q = 0; q < kFixZ; ++q) {
            const float inc = prefix + wave_inclusive_scan_f32(dv[q] * Al2);
            if (read_lane_f32(fast_exp2(inc), 0) == 0.f) dead = true;  // nothing reaches this tile, nor any later one
            if (q == z && !dead) cr = (tok0 + (k0 + q) * kQ + lane) < tend ? fast_exp2(inc) : 0.f;
            prefix = read_lane_f32(inc, kQ - 1);
        }
        // this workgroup's tile of the batch: k0 + z
        const int k = k0 + z;
        auto repair = [&](int pt, const bf16x8 (&et)[KS]) __attribute__((always_inline)) {
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const int tq = tok0 + k * kQ + 16 * tt + lr;  // this lane's token of the query block
                const float crt = __shfl(cr, 16 * tt + lr, 64);
                if (__ballot(crt != 0.f) == 0ull) continue;   // uniform per wave
                const bf16_t *crow = a.C + (row_of(tq) * a.G + g) * NS + 8 * lb;
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16(et[ks], *reinterpret_cast<const bf16x8 *>(crow + 32 * ks), acc);
                if (tq < tend && crt != 0.f) {
                    bf16x4 *yq = reinterpret_cast<bf16x4 *>(a.y + (size_t)tq * HP + (size_t)h * a.P + 16 * pt + 4 * lb);
                    const bf16x4 old = *yq;
                    bf16x4 out;
#pragma unroll
                    for (int e = 0; e < 4; ++e) out[e] = (bf16_t)((float)old[e] + crt * acc[e]);
                    *yq = out;
                }
            }
        };
        if (__ballot(cr != 0.f) != 0ull) {
            if (!have_e) {
#pragma unroll
                for (int q = 0; q < kMaxPT; ++q)
                    if (q < npt) load_e(wave + 4 * q, ef[q]);
                have_e = true;
            }
#pragma unroll
            for (int q = 0; q < kMaxPT; ++q)
                if (q < npt) repair(wave + 4 * q, ef[q]);
            for (int q = kMaxPT; q < npt; ++q) {
                bf16x8 et[KS];
                load_e(wave + 4 * q, et);
                repair(wave + 4 * q, et);
            }
        }
        if (dead) break;
    }
}

template <int NS, int NC, int NH, bool GATHER>
int launch(const SegArgs &a, hipStream_t st) {
    const int nunits = a.nseg * a.wg_per_seg;
    const size_t smem = sizeof(LdsS<NS, NC, NH>);
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&ssd_seg_kernel<NS, NC, NH, GATHER>), smem)) return STRD_EHIP;
    ssd_seg_kernel<NS, NC, NH, GATHER><<<xcd_grid(nunits), threads_for(NC, NH), smem, st>>>(a, nunits);
    if (a.nseg > 1) ssd_fix_kernel<NS, GATHER><<<dim3(a.nseg, a.H, kFixZ), kFixThreads, 0, st>>>(a);
    return launch_status();
}

// channels per workgroup / 32: the whole head when that divides, else one slab
int slabs_per_wg(int P) { return P % 64 == 0 ? 2 : 1; }
// heads per workgroup: two heads of one group share the B and C tiles when a head is one workgroup's
// worth of channels and the group has an even number of heads
int heads_per_wg(int H, int P, int G) { return P == 64 && (H / G) % 2 == 0 ? 2 : 1; }

}  // namespace

// How the sequence is cut: as many segments as it takes to give every CU a workgroup, each at least
// kMinSegSteps steps long (a shorter segment costs more in its prologue and at its seam than it gains).
void ssd_seg_plan(int T, int H, int P, int G, int *nseg, int *seg_steps) {
    constexpr int kMinSegSteps = 8, kCUs = 256;
    const int nsteps = (T + kQ - 1) / kQ;
    const int wg = H * (P / 32) / slabs_per_wg(P) / heads_per_wg(H, P, G);
    int s = wg >= kCUs ? 1 : (kCUs + wg - 1) / wg;
    s = max(1, min(s, nsteps / kMinSegSteps));
    const int per = (nsteps + s - 1) / s;
    *seg_steps = max(per, 1);
    *nseg = max(1, (nsteps + *seg_steps - 1) / *seg_steps);
}

size_t ssd_seg_ws(int T, int H, int P, int G, int n) {
    int nseg, seg_steps;
    ssd_seg_plan(T, H, P, G, &nseg, &seg_steps);
    if (nseg <= 1) return 0;
    return align_up((size_t)(nseg - 1) * H * P * n * sizeof(float), 256) + align_up((size_t)nseg * H * sizeof(float), 256);
}

// `rows` = number of rows of the source tensors (T for the dense call, N + M for the gather call)
bool ssd_seg_supported(int T, int rows, int H, int P, int G, int n, strd_dtype io) {
    const unsigned long long lim = 1ull << 32, r = (unsigned long long)(rows > T ? rows : T) + 2 * kQ;
    return io == STRD_BF16 && T >= 1 && (n == 64 || n == 128) && P % 32 == 0 && (long long)H * (P / 32) < (1 << 22) &&
           r * H * 4 < lim && H <= 65535;
}

// Whether this kernel or the one that walks the whole sequence in one workgroup per (head, 32
// channels) (ssd_mfma) is the faster one.  This kernel moves about half the bytes per token through
// a CU's copy path (B and C tiles serve the whole head) and fills the chip with few heads, but pays
// for its segments with a longer prologue and a second launch: it wins once a segment is long
// (measured: from about 32 steps at 128 heads), or when the other kernel would leave CUs idle.
bool ssd_seg_preferred(int T, int H, int P, int G) {
    int nseg, seg_steps;
    ssd_seg_plan(T, H, P, G, &nseg, &seg_steps);
    return nseg >= 2 && (seg_steps >= 32 || H * (P / 32) < 128);
}

int ssd_seg(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
            const float *S_in, void *y, float *S_out, const int32_t *idx, int N, int K, int T, int H, int P, int G, int n,
            void *ws, hipStream_t st) {
    SegArgs a;
    a.x = (const bf16_t *)x; a.dt = dt; a.A = A; a.B = (const bf16_t *)B; a.C = (const bf16_t *)C; a.D = D; a.S_in = S_in;
    a.y = (bf16_t *)y; a.S_out = S_out; a.idx = idx; a.N = N; a.K = K; a.T = T; a.H = H; a.P = P; a.G = G;
    ssd_seg_plan(T, H, P, G, &a.nseg, &a.seg_steps);
    const int nc = slabs_per_wg(P), nh = heads_per_wg(H, P, G);
    a.wg_per_seg = H * (P / 32) / nc / nh;
    a.lend = a.ltot = nullptr;
    if (a.nseg > 1) {
        if (!ws) return STRD_EWORKSPACE;
        a.lend = (float *)ws;
        a.ltot = (float *)((char *)ws + align_up((size_t)(a.nseg - 1) * H * P * n * sizeof(float), 256));
    }
#define STRD_SEG_LAUNCH(NS_, NC_, NH_)                                                 \
    return idx ? launch<NS_, NC_, NH_, true>(a, st) : launch<NS_, NC_, NH_, false>(a, st)
    if (n == 128 && nc == 2 && nh == 2) { STRD_SEG_LAUNCH(128, 2, 2); }
    if (n == 64 && nc == 2 && nh == 2) { STRD_SEG_LAUNCH(64, 2, 2); }
    if (n == 128 && nc == 2) { STRD_SEG_LAUNCH(128, 2, 1); }
    if (n == 128 && nc == 1) { STRD_SEG_LAUNCH(128, 1, 1); }
    if (n == 64 && nc == 2) { STRD_SEG_LAUNCH(64, 2, 1); }
    if (n == 64 && nc == 1) { STRD_SEG_LAUNCH(64, 1, 1); }
#undef STRD_SEG_LAUNCH
    return STRD_EUNSUPPORTED;
}

}  // namespace strd
