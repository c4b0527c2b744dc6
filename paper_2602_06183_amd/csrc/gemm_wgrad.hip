// Weight-gradient contractions of the fused step, eq. (5) dW2 = y2.T dY and eq. (8) dW1 = dy1.T X (Alg. 2 lines 3, 6):
//   C[f, n] = sum_t A[t, f] * G[t, n],  A = the V:N:M activation (y2 or dy1), G = dY or X, contraction over tokens.
// The 2:4 structure of A lies along the output rows here, so the structured-sparse matrix instruction does not apply;
// what the format still gives is that, inside a block of 64 tokens, only 4 of every 8 hidden units are non-zero.
// The producer (the V:N:M epilogue of gemm_v2.hip) therefore stores the transposed activation compacted to those
// rows ("atc": row 4 g + p of token block tb = hidden unit 8 g + colidx[tb, g, p]; [F / 2 rows, T tokens], blocked
// layout of common.hpp), which halves its bytes in HBM, in L2 and on the way into LDS.  This kernel runs dense
// v_mfma_f32_32x32x16_bf16 on a 256 (hidden) x 256 tile; a lane that needs hidden unit f looks up, once per
// 64-token stage, whether f is one of its group's four kept units (a bit mask per group, written by the producer;
// the position among the kept units is a population count) and reads either that compact row or a row of zeros
// kept at the end of the tile.  Same ring / barrier / LDS-DMA discipline as gemm_v2.hip: 3 stages of 64
// tokens (A 16 KB as two 32-token halves, G 32 KB as two halves, 8 private copies of the tile's 32 mask bytes).
#include "common.hpp"
#include "kernels.hpp"
#include "lds_dma.hpp"

namespace sffn {

namespace {

constexpr int kAHalf = 128 * 64 + 64;            // 128 compact rows x 32 tokens, then one row of zeros
constexpr int kABytes = 2 * kAHalf;
constexpr int kBHalf = 256 * 64;
constexpr int kBBytes = 2 * kBHalf;
constexpr int kStage = kABytes + kBBytes + 8 * 256;
constexpr int kStages = 3;
constexpr int kLoads = 2 + 4 + 1;                // LDS-DMA loads per wavefront per stage

}  // namespace

// Accumulators of one 128 x 64 wave tile -> bf16 output (one rounding; `alpha` = product of the operand scales of the fp8 form, 1 otherwise).
// ACC32: `out` is a float32 matrix of the same shape that the tile is ADDED to (gradient accumulation over the micro-batches of an
// optimizer step): out32 = out32 + alpha * sum, both in float32.
template <bool OUT_I_CONTIG, bool ACC32>
__device__ __forceinline__ void wgrad_store(f32x16 (&acc)[4][2], float alpha, unsigned char* smem, int wave, int lane, int i0, int j0, int F, int N,
                                            uint16_t* __restrict__ out, int64_t ldo) {
    constexpr int WM = 128, WN = 64, FM = 4, FN = 2;
    const int wm = wave >> 2, wn = wave & 3, l32 = lane & 31, lh = lane >> 5;
    if (ACC32 && OUT_I_CONTIG) {
        // out32[j * ldo + i]: a lane owns 4 consecutive i of one j; stage [32 j][64 i] through LDS so that HBM sees 256-byte row
        // segments in 16-byte accesses (read, add, write)
        float* out32 = reinterpret_cast<float*>(out);
        constexpr int EP = 64 * 4 + 16;
        unsigned char* scratch = smem + wave * (32 * EP);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int b = 0; b < FN; ++b) {
                const int f0 = i0 + wm * WM + h * 64, n0 = j0 + wn * WN + b * 32;
#pragma unroll
                for (int a2 = 0; a2 < 2; ++a2)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int a = 2 * h + a2;
                        *reinterpret_cast<float4*>(scratch + l32 * EP + (a2 * 32 + 8 * g + 4 * lh) * 4) =
                            make_float4(acc[a][b][4 * g] * alpha, acc[a][b][4 * g + 1] * alpha, acc[a][b][4 * g + 2] * alpha, acc[a][b][4 * g + 3] * alpha);
                    }
                wave_lds_sync();
                // all of the slab's old values are requested before the first sum is stored (a store would otherwise stand between the loads)
                float4 old[8];
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    const int row = p * 4 + (lane >> 4), ch = lane & 15;
                    const int j = n0 + row, i = f0 + ch * 4;
                    old[p] = (j < N && i < F) ? *reinterpret_cast<const float4*>(out32 + (int64_t)j * ldo + i) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    const int row = p * 4 + (lane >> 4), ch = lane & 15;
                    const int j = n0 + row, i = f0 + ch * 4;
                    if (j < N && i < F) {
                        const float4 add = *reinterpret_cast<const float4*>(scratch + row * EP + ch * 16);
                        *reinterpret_cast<float4*>(out32 + (int64_t)j * ldo + i) = make_float4(old[p].x + add.x, old[p].y + add.y, old[p].z + add.z, old[p].w + add.w);
                    }
                }
                wave_lds_sync();
            }
    } else if (ACC32) {
        // out32[i * ldo + j]: each 32-row slab goes through LDS, as in the bf16 form below, for 16-byte accesses on 256-byte row segments;
        // the products are rounded to float32 before they are staged, so the addition is never a fused multiply-add
        float* out32 = reinterpret_cast<float*>(out);
        constexpr int EP = WN * 4 + 16;
        unsigned char* scratch = smem + wave * (32 * EP);
#pragma unroll
        for (int a = 0; a < FM; ++a) {
#pragma unroll
            for (int b = 0; b < FN; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + 4 * lh + (r & 3);
                    *reinterpret_cast<float*>(scratch + row * EP + (b * 32 + l32) * 4) = acc[a][b][r] * alpha;
                }
            wave_lds_sync();
            float4 old[8];
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int row = p * 4 + (lane >> 4), ch = lane & 15;
                const int i = i0 + wm * WM + a * 32 + row, j = j0 + wn * WN + ch * 4;
                old[p] = (i < F && j < N) ? *reinterpret_cast<const float4*>(out32 + (int64_t)i * ldo + j) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int row = p * 4 + (lane >> 4), ch = lane & 15;
                const int i = i0 + wm * WM + a * 32 + row, j = j0 + wn * WN + ch * 4;
                if (i < F && j < N) {
                    const float4 add = *reinterpret_cast<const float4*>(scratch + row * EP + ch * 16);
                    *reinterpret_cast<float4*>(out32 + (int64_t)i * ldo + j) = make_float4(old[p].x + add.x, old[p].y + add.y, old[p].z + add.z, old[p].w + add.w);
                }
            }
            wave_lds_sync();
        }
    } else if (OUT_I_CONTIG) {
        // out[j * ldo + i]: a lane owns 4 consecutive i of one j; stage [j][i] through LDS (two halves of 64 i)
        // so that HBM sees 128-byte row segments
        constexpr int EP = 64 * 2 + 16;
        unsigned char* scratch = smem + wave * (WN * EP);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int f0 = i0 + wm * WM + h * 64, n0 = j0 + wn * WN;
#pragma unroll
            for (int a2 = 0; a2 < 2; ++a2)
#pragma unroll
                for (int b = 0; b < FN; ++b)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int a = 2 * h + a2, il = a2 * 32 + 8 * g + 4 * lh;
                        *reinterpret_cast<uint2*>(scratch + (b * 32 + l32) * EP + il * 2) =
                            make_uint2(f2bf2(acc[a][b][4 * g] * alpha, acc[a][b][4 * g + 1] * alpha), f2bf2(acc[a][b][4 * g + 2] * alpha, acc[a][b][4 * g + 3] * alpha));
                    }
            wave_lds_sync();
#pragma unroll
            for (int p = 0; p < WN / 8; ++p) {
                const int row = p * 8 + (lane >> 3), ch = lane & 7;
                const int j = n0 + row, i = f0 + ch * 8;
                if (j < N && i < F)
                    *reinterpret_cast<uint4*>(out + (int64_t)j * ldo + i) = *reinterpret_cast<const uint4*>(scratch + row * EP + ch * 16);
            }
            wave_lds_sync();
        }
    } else {
        // out[i * ldo + j]: transpose each 32-row slab through LDS for 16-byte row stores
        constexpr int EP = WN * 2 + 16;
        unsigned char* scratch = smem + wave * (32 * EP);
#pragma unroll
        for (int a = 0; a < FM; ++a) {
#pragma unroll
            for (int b = 0; b < FN; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + 4 * lh + (r & 3);
                    *reinterpret_cast<uint16_t*>(scratch + row * EP + (b * 32 + l32) * 2) = (uint16_t)f2bf(acc[a][b][r] * alpha);
                }
            wave_lds_sync();
#pragma unroll
            for (int p = 0; p < 32 * (WN / 8) / 64; ++p) {
                const int e = lane + 64 * p, row = e / (WN / 8), ch = e % (WN / 8);
                const int i = i0 + wm * WM + a * 32 + row, j = j0 + wn * WN + ch * 8;
                if (i < F && j < N)
                    *reinterpret_cast<uint4*>(out + (int64_t)i * ldo + j) = *reinterpret_cast<const uint4*>(scratch + row * EP + ch * 16);
            }
            wave_lds_sync();
        }
    }
}

template <bool OUT_I_CONTIG, bool ACC32>
__global__ void __launch_bounds__(512) wgrad_vnm_kernel(const uint16_t* __restrict__ atc, const uint8_t* __restrict__ kmask,
                                                       const uint16_t* __restrict__ G, int F, int N, int Ttot,
                                                       uint16_t* __restrict__ out, int64_t ldo, int tiles_m, int tiles_n,
                                                       GemmGroup grp) {
    constexpr int BM = 256, BN = 256, WM = 128, WN = 64, FM = 4, FN = 2;
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kStages * kStage];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int l32 = lane & 31, lh = lane >> 5;

    // workgroup -> tile: an XCD gets a run of consecutive logical ids, which walk bands of 4 tile rows
    int L;
    {
        const int n = gridDim.x, pid = blockIdx.x, per = n >> 3;
        L = (pid < per * 8) ? (pid & 7) * per + (pid >> 3) : pid;
    }
    int k_base = 0, K = Ttot;                     // grouped: every expert contracts over its own token segment
    if (grp.n) {
        const int per = tiles_m * tiles_n, e = L / per;
        L -= e * per;
        k_base = grp.seg[e];
        K = grp.seg[e + 1] - k_base;
        out += e * grp.out_stride * (ACC32 ? 2 : 1);          // (float32 elements are two uint16_t wide)
    }
    int tm, tn;
    {
        constexpr int GROUP = SFFN_TILE_GROUP;
        const int width = GROUP * tiles_n, group = L / width, first = group * GROUP;
        const int gsz = (tiles_m - first) < GROUP ? (tiles_m - first) : GROUP;
        tm = first + (L % width) % gsz;
        tn = (L % width) / gsz;
    }
    const int i0 = tm * BM, j0 = tn * BN;
    const int KC = Ttot / 32;                     // 32-token chunks per row of the blocked operands

    // ---- wave-uniform sources of the DMA loads (tile 0 of the k loop) and per-lane offsets.  Rows past the
    //      matrix edge are clamped into it: they only feed outputs that are never stored. ------------------
    uint64_t a_base[2], b_base[4], c_base;
    const int rb = lane >> 2;
    const uint32_t blk_lane = (uint32_t)(rb * 32 + ((lane & 3) ^ ((rb >> 2) & 3)) * 8) * 2;   // chunk swizzle, see gemm_v2.hip
    {
        int cr = i0 / 2 + wave * 16; cr = cr < F / 2 ? cr : F / 2 - 16;
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) a_base[kc] = uniform64(atc + (((int64_t)(cr >> 4) * KC + k_base / 32 + kc) << 9));
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const int bk = wave * 4 + n, h = bk >> 4;
            int gr = j0 + (bk & 15) * 16; gr = gr < N ? gr : N - 16;
            b_base[n] = uniform64(G + (((int64_t)(gr >> 4) * KC + k_base / 32 + h) << 9));
        }
        c_base = uniform64(kmask + (int64_t)(k_base / 64) * (F / 8));
    }
    // mask bytes of the tile's 32 groups of 8 hidden units (lanes 0-7 bring 4 each, the others repeat them); every
    // wavefront fetches its own copy
    uint32_t c_lane;
    {
        int g = i0 / 8 + 4 * (lane & 7); g = g < F / 8 ? g : F / 8 - 4;
        c_lane = (uint32_t)g;
    }
    const uint32_t c_kstep = (uint32_t)(F / 8);

    auto issue_half = [&](int kt, int stage, int h) {
        unsigned char* sa = smem + stage * kStage;
        unsigned char* sb = sa + kABytes;
        unsigned char* sc = sb + kBBytes;
        const uint32_t o = blk_lane + (uint32_t)kt * 2048;      // k position in the per-lane offset; bases stay in SGPRs
        if (h == 0) {
            dma4(c_base, c_lane + (uint32_t)kt * c_kstep, sc + wave * 256);     // first: the look-up wants it earliest
            dma16(a_base[0], o, sa + wave * 1024);
            dma16(a_base[1], o, sa + kAHalf + wave * 1024);
            dma16(b_base[0], o, sb + (wave * 4 + 0) * 1024);
            dma16(b_base[1], o, sb + (wave * 4 + 1) * 1024);
        } else {
            dma16(b_base[2], o, sb + (wave * 4 + 2) * 1024);
            dma16(b_base[3], o, sb + (wave * 4 + 3) * 1024);
        }
    };

    // ---- fragment reads.  Sub-step s (16 tokens) of a stage lives in half s / 2 at chunk pair s % 2. ----
    int b_off[FN];
#pragma unroll
    for (int b = 0; b < FN; ++b) {
        const int row = wn * WN + b * 32 + l32;
        b_off[b] = kABytes + row * 64 + ((lh ^ ((row >> 2) & 3)) << 4);
    }
    // hidden unit of fragment a in this lane: f = i0 + wm * 128 + a * 32 + l32 -> group wm * 16 + a * 4 + l32 / 8 of the tile,
    // column l32 % 8 of the group.  a_off[a] = its row in a half-tile (or the zero row), set per stage by lookup().
    // a_off[a][0 / 1] = LDS address of its row (or of the zero row) for the even / odd 16-token sub-steps of a half-tile
    int a_off[FM][2], a_next[FM][2];
    const uint32_t col = l32 & 7, below = (1u << col) - 1u;
    // the zero row is read at the chunk pair the lanes of the same 16-lane phase do not use for kept rows (no bank conflict)
    const int zero_row = 128 * 64 + ((lh ^ (l32 >> 3) ^ 2) << 4);
    uint32_t mk[FM];
    auto lookup_read = [&](int stage) {
        const unsigned char* sc = smem + stage * kStage + kABytes + kBBytes + wave * 256;
#pragma unroll
        for (int a = 0; a < FM; ++a) mk[a] = sc[wm * 16 + a * 4 + (l32 >> 3)];
    };
    auto lookup = [&](int stage) {
        const int sa = stage * kStage;
#pragma unroll
        for (int a = 0; a < FM; ++a) {
            const int gl = wm * 16 + a * 4 + (l32 >> 3);
            const int row = gl * 4 + __builtin_popcount(mk[a] & below);                   // (row >> 2) & 3 == l32 >> 3
            const int off = ((mk[a] >> col) & 1u) ? row * 64 + ((lh ^ (l32 >> 3)) << 4) : zero_row;
            a_next[a][0] = sa + off;
            a_next[a][1] = sa + (off ^ 32);
        }
    };
    struct FragSet { Frag8 a[FM]; Frag8 b[FN]; };
    auto read_a = [&](FragSet& f, const unsigned char* st, int s, int a) {
        (void)st;
        f.a[a].u = *reinterpret_cast<const uint4*>(smem + a_off[a][s & 1] + (s >> 1) * kAHalf);
    };
    auto read_b = [&](FragSet& f, const unsigned char* st, int s, int b) {
        f.b[b].u = *reinterpret_cast<const uint4*>(st + (s >> 1) * kBHalf + (b_off[b] ^ (32 * (s & 1))));
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;
    auto mma_row = [&](const FragSet& f, int a) {
#pragma unroll
        for (int b = 0; b < FN; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[a].v, f.b[b].v, acc[a][b], 0, 0, 0);
    };
#define SB() __builtin_amdgcn_sched_barrier(0)

    const int nk = K / 64;              // 0 for an expert without tokens: its gradient is zero
    if (nk > 0) {
        // rows of zeros behind both half-tiles of every stage (never touched by the DMA)
        if (tid < kStages * 2 * 16) *reinterpret_cast<uint32_t*>(smem + (tid >> 5) * kStage + ((tid >> 4) & 1) * kAHalf + 128 * 64 + (tid & 15) * 4) = 0u;
#pragma unroll
        for (int p = 0; p < kStages; ++p) { issue_half(p < nk ? p : nk - 1, p, 0); issue_half(p < nk ? p : nk - 1, p, 1); }
        wait_vmcnt<(kStages - 1) * kLoads>();
        __syncthreads();
        FragSet P, Q;
        lookup_read(0);
        lookup(0);
#pragma unroll
        for (int a = 0; a < FM; ++a) { a_off[a][0] = a_next[a][0]; a_off[a][1] = a_next[a][1]; read_a(P, smem, 0, a); }
#pragma unroll
        for (int b = 0; b < FN; ++b) read_b(P, smem, 0, b);
        int stage = 0;
        // One step = one stage = four sub-steps of eight matrix instructions; the fragments of a sub-step are read
        // while the matrix cores work on the one before.  Before the last sub-step every wavefront has read all of
        // the stage (barrier), which is then refilled with the tile three steps ahead while the next stage's rows
        // are looked up and its first fragments fetched.
        for (int kt = 0; kt < nk; ++kt) {
            const int nxt = (kt + kStages < nk) ? kt + kStages : nk - 1;
            const int next_stage = (stage + 1 == kStages) ? 0 : stage + 1;
            const unsigned char* st = smem + stage * kStage;
            const unsigned char* sn = smem + next_stage * kStage;
            mma_row(P, 0); SB();
            read_a(Q, st, 1, 0); read_a(Q, st, 1, 1); read_b(Q, st, 1, 0); SB();
            mma_row(P, 1); SB();
            read_a(Q, st, 1, 2); read_a(Q, st, 1, 3); read_b(Q, st, 1, 1); SB();
            mma_row(P, 2); SB();
            mma_row(P, 3); SB();
            mma_row(Q, 0); SB();
            read_a(P, st, 2, 0); read_a(P, st, 2, 1); read_b(P, st, 2, 0); SB();
            mma_row(Q, 1); SB();
            read_a(P, st, 2, 2); read_a(P, st, 2, 3); read_b(P, st, 2, 1); SB();
            // the next tile's mask bytes were the first load of its batch: all but kLoads - 1 of that batch and
            // the batch after it may still be in flight
            wait_vmcnt<(kStages - 2) * kLoads + kLoads - 1>();
            lookup_read(next_stage); SB();
            mma_row(Q, 2); SB();
            mma_row(Q, 3); SB();
            mma_row(P, 0); SB();
            read_a(Q, st, 3, 0); read_a(Q, st, 3, 1); read_b(Q, st, 3, 0); SB();
            mma_row(P, 1); SB();
            read_a(Q, st, 3, 2); read_a(Q, st, 3, 3); read_b(Q, st, 3, 1); SB();
            lookup(next_stage); SB();
            mma_row(P, 2); SB();
            mma_row(P, 3); SB();
            wait_vmcnt_lgkm0<(kStages - 2) * kLoads>();      // Q is here, tile kt + 1 has landed (this wavefront's part)
            __builtin_amdgcn_s_barrier();
            SB();
#pragma unroll
            for (int a = 0; a < FM; ++a) { a_off[a][0] = a_next[a][0]; a_off[a][1] = a_next[a][1]; }
            mma_row(Q, 0); SB();
            read_a(P, sn, 0, 0); read_a(P, sn, 0, 1); read_b(P, sn, 0, 0); SB();
            mma_row(Q, 1); SB();
            read_a(P, sn, 0, 2); read_a(P, sn, 0, 3); read_b(P, sn, 0, 1); SB();
            issue_half(nxt, stage, 0); SB();
            mma_row(Q, 2); SB();
            issue_half(nxt, stage, 1); SB();
            mma_row(Q, 3); SB();
            stage = next_stage;
        }
        wait_vmcnt<0>();
    }
#undef SB
    __syncthreads();

    wgrad_store<OUT_I_CONTIG, ACC32>(acc, 1.0f, smem, wave, lane, i0, j0, F, N, out, ldo);
}

// The same contraction on E4M3 codes (the fp8 step with SFFN_FLAG_FP8_WGRAD): atc and G hold one code per element, in the blocked layout
// with a pair of codes per 2-byte element, so one 64-byte chunk of a row is exactly one 64-token block.  v_mfma_scale_f32_32x32x64_f8f6f4 with
// unit scales contracts one such block per instruction (measured: lane l supplies k 32 (l / 32) .. + 31 of row / column l % 32 in both
// operands; 2x the bf16 rate).  A stage of the ring is therefore ONE token block: compact A 8 KB + a row of zeros, G 16 KB, 8 private copies
// of the block's 32 mask bytes; 5 stages; per stage four rows of two matrix instructions, the A fragments read one row ahead, the G
// fragments one stage ahead.  out = bf16(alpha * sum), alpha = product of the two tensor scales.
namespace {
constexpr int k8A = 128 * 64 + 64;               // 128 compact rows x 64 tokens, then one row of zeros
constexpr int k8B = 256 * 64;
constexpr int k8Stage = k8A + k8B + 8 * 256;
constexpr int k8Stages = 5;
constexpr int k8Loads = 1 + 1 + 2;               // mask, A block, two G blocks per wavefront and stage
}  // namespace

template <bool OUT_I_CONTIG, bool ACC32>
__global__ void __launch_bounds__(512) wgrad_vnm_fp8_kernel(const uint16_t* __restrict__ atc, const uint8_t* __restrict__ kmask,
                                                           const uint16_t* __restrict__ G, int F, int N, int Ttot, float alpha,
                                                           uint16_t* __restrict__ out, int64_t ldo, int tiles_m, int tiles_n, GemmGroup grp) {
    constexpr int BM = 256, BN = 256, WM = 128, WN = 64, FM = 4, FN = 2;
    __shared__ __attribute__((aligned(1024))) unsigned char smem[k8Stages * k8Stage];
    static_assert(8 * 64 * (64 * 2 + 16) <= sizeof(smem), "epilogue scratch must fit");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int l32 = lane & 31, lh = lane >> 5;
    int L;
    {
        const int n = gridDim.x, pid = blockIdx.x, per = n >> 3;
        L = (pid < per * 8) ? (pid & 7) * per + (pid >> 3) : pid;
    }
    int k_base = 0, K = Ttot;                     // grouped: every expert contracts over its own token segment
    if (grp.n) {
        const int per = tiles_m * tiles_n, e = L / per;
        L -= e * per;
        k_base = grp.seg[e];
        K = grp.seg[e + 1] - k_base;
        out += e * grp.out_stride * (ACC32 ? 2 : 1);          // (float32 elements are two uint16_t wide)
    }
    int tm, tn;
    {
        constexpr int GROUP = SFFN_TILE_GROUP;
        const int width = GROUP * tiles_n, group = L / width, first = group * GROUP;
        const int gsz = (tiles_m - first) < GROUP ? (tiles_m - first) : GROUP;
        tm = first + (L % width) % gsz;
        tn = (L % width) / gsz;
    }
    const int i0 = tm * BM, j0 = tn * BN;
    const int KC = Ttot / 64;                     // 64-token chunks (64 bytes) per row of the blocked operands

    uint64_t a_base, b_base[2], c_base;
    const int rb = lane >> 2;
    const uint32_t blk_lane = (uint32_t)(rb * 32 + ((lane & 3) ^ ((rb >> 2) & 3)) * 8) * 2;   // chunk swizzle, as in the bf16 kernel
    {
        int cr = i0 / 2 + wave * 16; cr = cr < F / 2 ? cr : F / 2 - 16;
        a_base = uniform64(atc + (((int64_t)(cr >> 4) * KC + k_base / 64) << 9));
#pragma unroll
        for (int n = 0; n < 2; ++n) {
            int gr = j0 + (wave * 2 + n) * 16; gr = gr < N ? gr : N - 16;
            b_base[n] = uniform64(G + (((int64_t)(gr >> 4) * KC + k_base / 64) << 9));
        }
        c_base = uniform64(kmask + (int64_t)(k_base / 64) * (F / 8));
    }
    uint32_t c_lane;
    {
        int g = i0 / 8 + 4 * (lane & 7); g = g < F / 8 ? g : F / 8 - 4;
        c_lane = (uint32_t)g;
    }
    const uint32_t c_kstep = (uint32_t)(F / 8);
    auto issue = [&](int kt, int stage) {
        unsigned char* sa = smem + stage * k8Stage;
        const uint32_t o = blk_lane + (uint32_t)kt * 1024;
        dma4(c_base, c_lane + (uint32_t)kt * c_kstep, sa + k8A + k8B + wave * 256);     // first: the look-up wants it earliest
        dma16(a_base, o, sa + wave * 1024);
        dma16(b_base[0], o, sa + k8A + (wave * 2 + 0) * 1024);
        dma16(b_base[1], o, sa + k8A + (wave * 2 + 1) * 1024);
    };

    // fragment reads: a lane wants the 32 bytes k 32 lh .. + 31 of its row = 16-byte chunks 2 lh, 2 lh + 1 (slot = chunk ^ ((row >> 2) & 3))
    int b_off[FN];
#pragma unroll
    for (int b = 0; b < FN; ++b) {
        const int row = wn * WN + b * 32 + l32;
        b_off[b] = k8A + row * 64 + (((2 * lh) ^ ((row >> 2) & 3)) << 4);
    }
    int a_off[FM], a_next[FM];
    const uint32_t col = l32 & 7, below = (1u << col) - 1u;
    const int zero_row = 128 * 64 + (((2 * lh) ^ (l32 >> 3) ^ 2) << 4);
    uint32_t mk[FM];
    auto lookup_read = [&](int stage) {
        const unsigned char* sc = smem + stage * k8Stage + k8A + k8B + wave * 256;
#pragma unroll
        for (int a = 0; a < FM; ++a) mk[a] = sc[wm * 16 + a * 4 + (l32 >> 3)];
    };
    auto lookup = [&](int stage) {
        const int sa = stage * k8Stage;
#pragma unroll
        for (int a = 0; a < FM; ++a) {
            const int gl = wm * 16 + a * 4 + (l32 >> 3);
            const int row = gl * 4 + __builtin_popcount(mk[a] & below);                   // (row >> 2) & 3 == l32 >> 3
            a_next[a] = sa + (((mk[a] >> col) & 1u) ? row * 64 + (((2 * lh) ^ (l32 >> 3)) << 4) : zero_row);
        }
    };
    auto read_a = [&](Frag16& f, int off) {
        f.u[0] = *reinterpret_cast<const uint4*>(smem + off);
        f.u[1] = *reinterpret_cast<const uint4*>(smem + (off ^ 16));
    };
    auto read_b = [&](Frag16& f, const unsigned char* st, int b) {
        f.u[0] = *reinterpret_cast<const uint4*>(st + b_off[b]);
        f.u[1] = *reinterpret_cast<const uint4*>(st + (b_off[b] ^ 16));
    };
    f32x16 acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;
    auto mma_row = [&](const Frag16& fa, const Frag16 (&fb)[FN], int a) {
#pragma unroll
        for (int b = 0; b < FN; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa.q, fb[b].q, acc[a][b], 0, 0, 0, 0x7F, 0, 0x7F);   // fp8 x fp8, scales 2^0
    };
#define SB() __builtin_amdgcn_sched_barrier(0)
    const int nk = K / 64;                // 0 for an expert without tokens: its gradient is zero
    if (nk > 0) {
        if (tid < k8Stages * 16) *reinterpret_cast<uint32_t*>(smem + (tid >> 4) * k8Stage + 128 * 64 + (tid & 15) * 4) = 0u;   // the rows of zeros
#pragma unroll
        for (int p = 0; p < k8Stages; ++p) issue(p < nk ? p : nk - 1, p);
        wait_vmcnt<(k8Stages - 1) * k8Loads>();
        __syncthreads();
        Frag16 A0, A1, B0[FN], B1[FN];
        lookup_read(0);
        lookup(0);
#pragma unroll
        for (int a = 0; a < FM; ++a) a_off[a] = a_next[a];
        read_a(A0, a_off[0]);
#pragma unroll
        for (int b = 0; b < FN; ++b) read_b(B0[b], smem, b);
        int stage = 0;
        // One step = one token block; two steps per loop trip so that the two G fragment sets alternate by name.
        auto step = [&](int kt, Frag16 (&Bc)[FN], Frag16 (&Bn)[FN]) {
            const int nxt = (kt + k8Stages < nk) ? kt + k8Stages : nk - 1;
            const int next_stage = (stage + 1 == k8Stages) ? 0 : stage + 1;
            const unsigned char* sn = smem + next_stage * k8Stage;
            read_a(A1, a_off[1]); SB();
            mma_row(A0, Bc, 0); SB();
            read_a(A0, a_off[2]); SB();
            mma_row(A1, Bc, 1); SB();
            read_a(A1, a_off[3]); SB();
            // the next block's mask bytes were the first load of its batch
            wait_vmcnt<(k8Stages - 2) * k8Loads + k8Loads - 1>();
            lookup_read(next_stage); SB();
            mma_row(A0, Bc, 2); SB();
            wait_vmcnt_lgkm0<(k8Stages - 2) * k8Loads>();      // my reads of this stage are done, block kt + 1 has landed (this wavefront's part)
            __builtin_amdgcn_s_barrier();
            SB();
            issue(nxt, stage); SB();
            lookup(next_stage); SB();
#pragma unroll
            for (int a = 0; a < FM; ++a) a_off[a] = a_next[a];
            read_a(A0, a_off[0]);
#pragma unroll
            for (int b = 0; b < FN; ++b) read_b(Bn[b], sn, b);
            SB();
            mma_row(A1, Bc, 3); SB();
            stage = next_stage;
        };
        int kt = 0;
        for (; kt + 1 < nk; kt += 2) { step(kt, B0, B1); step(kt + 1, B1, B0); }
        if (kt < nk) step(kt, B0, B1);
        wait_vmcnt<0>();
    }
#undef SB
    __syncthreads();
    wgrad_store<OUT_I_CONTIG, ACC32>(acc, alpha, smem, wave, lane, i0, j0, F, N, out, ldo);
}

hipError_t launch_wgrad_vnm_fp8(const uint8_t* atc, const uint8_t* kmask, const uint8_t* Gq, float alpha, int64_t F, int64_t N, int64_t T,
                                int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp, bool acc32) {
    if (T % 64 != 0 || T <= 0) return hipErrorInvalidValue;
    const int tiles_m = (int)((F + 255) / 256), tiles_n = (int)((N + 255) / 256);
    const GemmGroup gg = grp ? *grp : GemmGroup();
    if (gg.n && (gg.n > GemmGroup::kMaxExperts || gg.role != 2)) return hipErrorInvalidValue;
    dim3 grid((unsigned)(tiles_m * tiles_n * (gg.n ? gg.n : 1)));
    const uint16_t* a = reinterpret_cast<const uint16_t*>(atc);
    const uint16_t* g = reinterpret_cast<const uint16_t*>(Gq);
    if (out_i_contig && acc32)
        hipLaunchKernelGGL((wgrad_vnm_fp8_kernel<true, true>), grid, dim3(512), 0, s, a, kmask, g, (int)F, (int)N, (int)T, alpha, out, ldo, tiles_m, tiles_n, gg);
    else if (out_i_contig)
        hipLaunchKernelGGL((wgrad_vnm_fp8_kernel<true, false>), grid, dim3(512), 0, s, a, kmask, g, (int)F, (int)N, (int)T, alpha, out, ldo, tiles_m, tiles_n, gg);
    else if (acc32)
        hipLaunchKernelGGL((wgrad_vnm_fp8_kernel<false, true>), grid, dim3(512), 0, s, a, kmask, g, (int)F, (int)N, (int)T, alpha, out, ldo, tiles_m, tiles_n, gg);
    else
        hipLaunchKernelGGL((wgrad_vnm_fp8_kernel<false, false>), grid, dim3(512), 0, s, a, kmask, g, (int)F, (int)N, (int)T, alpha, out, ldo, tiles_m, tiles_n, gg);
    return hipGetLastError();
}

hipError_t launch_wgrad_vnm(const uint16_t* atc, const uint8_t* kmask, const uint16_t* G, int64_t F, int64_t N, int64_t T,
                            int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp, bool acc32) {
    const int tiles_m = (int)((F + 255) / 256), tiles_n = (int)((N + 255) / 256);
    const GemmGroup g = grp ? *grp : GemmGroup();
    if (g.n && (g.n > GemmGroup::kMaxExperts || g.role != 2)) return hipErrorInvalidValue;
    dim3 grid((unsigned)(tiles_m * tiles_n * (g.n ? g.n : 1)));
    if (out_i_contig && acc32)
        hipLaunchKernelGGL((wgrad_vnm_kernel<true, true>), grid, dim3(512), 0, s, atc, kmask, G, (int)F, (int)N, (int)T, out, ldo, tiles_m, tiles_n, g);
    else if (out_i_contig)
        hipLaunchKernelGGL((wgrad_vnm_kernel<true, false>), grid, dim3(512), 0, s, atc, kmask, G, (int)F, (int)N, (int)T, out, ldo, tiles_m, tiles_n, g);
    else if (acc32)
        hipLaunchKernelGGL((wgrad_vnm_kernel<false, true>), grid, dim3(512), 0, s, atc, kmask, G, (int)F, (int)N, (int)T, out, ldo, tiles_m, tiles_n, g);
    else
        hipLaunchKernelGGL((wgrad_vnm_kernel<false, false>), grid, dim3(512), 0, s, atc, kmask, G, (int)F, (int)N, (int)T, out, ldo, tiles_m, tiles_n, g);
    return hipGetLastError();
}

}  // namespace sffn
