// rotate_quant with dense rotation blocks: G_t(X) = (X . Delta) . BlockDiag(R_1 .. R_nb) (Eq. 10
// with the blocks of the BlockDiag equation of Sec. 3.2 as arbitrary orthogonal 128 x 128 matrices,
// e.g. the greedy ones of Eq. 6-7), followed by the per-token symmetric int8 quantiser.
//
// The rotation is a real contraction (128 x 128 per block and token), so it runs on the matrix
// cores: out^T = R'^T . X^T per block with R' = diag(d_b) . R_b, v_mfma_f32_16x16x32_bf16.
//   B operand: the raw bf16 activations, 16 tokens x 32 channels per instruction (a lane's 16-byte
//              load is its operand: no conversion, no LDS).
//   A operand: R'^T split EXACTLY into three bf16 pieces (8 + 8 + 8 mantissa bits; products with
//              bf16 activations are exact in fp32), prepared once per rotation in the fragment
//              order of the instruction.  The rows of an A tile are chosen so that a lane ends up
//              with 32 consecutive output channels of one token: tile t, row 4g + j holds output
//              channel 32 g + 4 t + j.
// A wave rotates whole blocks of one group of 16 * TT tokens; the token maximum crosses the
// workgroup through LDS, then the wave quantises and stores 32 bytes per lane and block.  The A pieces (96 KB per block) stream from L2;
// with TT = 2 every piece load feeds two instructions.
#include "device_utils.h"
#include "trdq_internal.h"

namespace trdq {

namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kPiecesPerBlock = 3 * 4 * 8 * 64;       // 16-byte fragments per block: piece, k-step, tile, lane

// pieces[(((b * 3 + p) * 4 + s) * 8 + t) * 64 + lane] = eight bf16: piece p of
//   d[b*128 + k] * R_b[k][c],  k = 32 s + 8 (lane >> 4) + e (e = 0..7),  c = 32 (r >> 2) + 4 t + (r & 3), r = lane & 15
__global__ __launch_bounds__(256) void rotation_pieces_kernel(const float *__restrict__ R, const float *__restrict__ diag,
                                                              uint16_t *__restrict__ pieces)
{
    const int b = blockIdx.y;
    const int idx = blockIdx.x * 256 + threadIdx.x;     // 0 .. 16383: (s, t, lane, e)
    const int e = idx & 7, lane = (idx >> 3) & 63, t = (idx >> 9) & 7, s = idx >> 12;
    const int r = lane & 15, g = lane >> 4;
    const int k = 32 * s + 8 * g + e;
    const int c = 32 * (r >> 2) + 4 * t + (r & 3);
    float v = R[((size_t)b * kBlock + k) * kBlock + c];
    if (diag) v *= diag[b * kBlock + k];
    // exact three-way split by truncation
    const uint32_t hi = __float_as_uint(v) & 0xFFFF0000u;
    const float r1 = v - __uint_as_float(hi);
    const uint32_t mid = __float_as_uint(r1) & 0xFFFF0000u;
    const float r2 = r1 - __uint_as_float(mid);
    const uint32_t lo = __float_as_uint(r2) & 0xFFFF0000u;
    const size_t base = (size_t)b * kPiecesPerBlock * 8;
    const size_t off = ((size_t)(s * 8 + t) * 64 + lane) * 8 + e;
    pieces[base + off] = (uint16_t)(hi >> 16);
    pieces[base + (size_t)1 * 4 * 8 * 64 * 8 + off] = (uint16_t)(mid >> 16);
    pieces[base + (size_t)2 * 4 * 8 * 64 * 8 + off] = (uint16_t)(lo >> 16);
}

// One block of one token group: out[tt][t][j] = rotated channel 32 g + 4 t + j of token tile tt's
// token l16 (this lane), amax[tt] = running maximum of |out|.  The A fragments (three pieces x four
// k-steps per tile) are requested one chunk ahead of the products; the scheduling barriers keep the
// compiler from requesting all 96 at once (which would not fit the register file) and from sinking
// the requests to just before their use (which would expose every load's latency).
template <int TT>
__device__ __forceinline__ void rotate_block_dense(const uint16_t *__restrict__ X, int64_t M, int64_t ldx,
                                                   const uint4 *__restrict__ pieces, int b, int64_t tok0, int lane,
                                                   float (&out)[TT][8][4], float (&amax)[TT])
{
    const int l16 = lane & 15, g = lane >> 4;
    // B operands: token tile tt, k-step s: channels b*128 + 32 s + 8 g .. + 7 of token l16
    v8bf xf[TT][4];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        int64_t token = tok0 + tt * 16 + l16;
        if (token >= M) token = M - 1;                  // a repeated row: its results are not stored
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            union { uint4 u; v8bf v; } ld;
            ld.u = *reinterpret_cast<const uint4 *>(X + token * ldx + b * kBlock + 32 * s + 8 * g);
            xf[tt][s] = ld.v;
        }
    }
    // (the offset passes through an empty assembly statement: where a wave keeps its block for every
    // token group the fragment loads would otherwise be hoisted out of the group loop, all 96 of them)
    int lane_off = lane;
    asm volatile("" : "+v"(lane_off));
    const uint4 *pb = pieces + (size_t)b * kPiecesPerBlock + lane_off;
    // The 96 fragments go through a two-deep ring of chunks of six (half a tile: k-steps and pieces in the
    // order they are multiplied, smallest piece first): chunk i + 1 is requested, then chunk i multiplied.
    constexpr int CH = 6, NCH = 12 / CH;
    uint4 fa[2][CH];
    auto request = [&](uint4 (&f)[CH], int i) {          // chunk i: tile i / NCH, fragments q = 11 - CH (i % NCH) - e
        const int t = i / NCH, q0 = 11 - CH * (i % NCH);
#pragma unroll
        for (int e = 0; e < CH; ++e) f[e] = pb[((q0 - e) * 8 + t) * 64];      // q = piece * 4 + k-step
    };
    request(fa[0], 0);
    v4f acc[TT];
#pragma unroll
    for (int i = 0; i < 8 * NCH; ++i) {
        if (i + 1 < 8 * NCH) request(fa[(i + 1) & 1], i + 1);
        __builtin_amdgcn_sched_barrier(0);      // the requests go out before this chunk's products, not after them
        const int t = i / NCH, q0 = 11 - CH * (i % NCH);
        if (i % NCH == 0) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) acc[tt] = v4f{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int e = 0; e < CH; ++e) {
            union { uint4 u; v8bf v; } a;
            a.u = fa[i & 1][e];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, xf[tt][(q0 - e) & 3], acc[tt], 0, 0, 0);
        }
        if (i % NCH == NCH - 1) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    out[tt][t][jj] = acc[tt][jj];
                    amax[tt] = fmaxf(amax[tt], fabsf(acc[tt][jj]));
                }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// 32 codes of one token and block -> 32 bytes at Xq[token][b*128 + 32 g]
__device__ __forceinline__ void store_codes_dense(const float (&o)[8][4], float inv, int8_t *dst8)
{
    uint32_t c[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
        c[t] = pack4_low_bytes(quant_bits(o[t][0], inv), quant_bits(o[t][1], inv),
                               quant_bits(o[t][2], inv), quant_bits(o[t][3], inv));
    uint4 *dst = reinterpret_cast<uint4 *>(dst8);
    dst[0] = make_uint4(c[0], c[1], c[2], c[3]);
    dst[1] = make_uint4(c[4], c[5], c[6], c[7]);
}

// A wave has one block (nb <= waves <= 12) and keeps its results in registers across the exchange of
// the token maxima.  Wider rows take the block-resident kernels further down.
template <int TT>
__global__ __launch_bounds__(768) void rotate_quant_dense_kernel(
    const uint16_t *__restrict__ X, int64_t M, int nb, int64_t ldx, const uint4 *__restrict__ pieces,
    int8_t *__restrict__ Xq, float *__restrict__ sx)
{
    extern __shared__ float amax_s[];                   // [2][nw][16 * TT]
    const int K = nb * kBlock;
    const int nw = blockDim.x >> 6;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    constexpr int TOK = 16 * TT;
    const int64_t groups = (M + TOK - 1) / TOK;
    int parity = 0;

    for (int64_t tg = blockIdx.x; tg < groups; tg += gridDim.x) {
        const int64_t tok0 = tg * TOK;
        float out[TT][8][4];
        float amax[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) amax[tt] = 0.0f;
        if (wave < nb) rotate_block_dense<TT>(X, M, ldx, pieces, wave, tok0, lane, out, amax);
        // token maximum: over the four lane groups, then over the waves
        float *const am = amax_s + parity * nw * TOK;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            amax[tt] = fmaxf(amax[tt], __shfl_xor(amax[tt], 16));
            amax[tt] = fmaxf(amax[tt], __shfl_xor(amax[tt], 32));
            if (g == 0) am[wave * TOK + tt * 16 + l16] = amax[tt];
        }
        __syncthreads();
        parity ^= 1;        // the next group writes the other buffer: one barrier per group
        float inv[TT];
        bool token_ok[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            float a = 0.0f;
            for (int w = 0; w < nw; ++w) a = fmaxf(a, am[w * TOK + tt * 16 + l16]);
            const int64_t token = tok0 + tt * 16 + l16;
            token_ok[tt] = token < M;
            inv[tt] = a > 0.0f ? 127.0f / a : 0.0f;
            if (wave == 0 && g == 0 && token_ok[tt]) sx[token] = a / 127.0f;
        }
        if (wave < nb) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                if (token_ok[tt])
                    store_codes_dense(out[tt], inv[tt], Xq + (tok0 + tt * 16 + l16) * K + wave * kBlock + 32 * g);
        }
    }
}

// ---- wide rows: a workgroup per block, its pieces resident in LDS -----------------------------
// Rows wider than 12 blocks do not fit the kernel above (a wave per block, results kept in
// registers).  Here a workgroup of eight waves takes ONE block, copies its pieces to LDS once and
// walks its share of the token tiles, TT at a time per wave (every LDS fragment read feeds TT
// matrix instructions); the activation fragments come straight from global memory, each wave its
// own tokens, one group of tiles ahead.  The token maximum spans blocks, i.e. workgroups, so there
// are two passes: kSinkMaxima merges |out| maxima into sx with atomic maxima on the bit patterns
// (non-negative floats order like integers; sx cleared before), kSinkCodes repeats the products,
// quantises and stores; a last kernel turns the maxima in sx into scales.
//
// The same kernel carries Eq. 10 with both rotations dense for wide rows, in three launches around a
// workspace T of once-rotated values, float32, CHANNEL-major ([K][ldt], ldt = tokens rounded up to 32):
//   kSinkRows          first rotation; the operands of the matrix instruction trade places, so that a lane
//                      ends up with four consecutive tokens of one channel and stores them as 16 bytes of T;
//   GATHER + kSinkMaxima / kSinkCodes
//                      second rotation; a lane's operand element k of a k-step is T[perm[b*128 + k]][token]
//                      (a 4-byte load; the 16 tokens of a lane row are 64 consecutive bytes; the 128 row
//                      numbers wait in LDS), float32, so it is split exactly into three bf16 pieces like the
//                      rotation itself, and the product takes the six piece pairs down to 2^-24 of |r||t|
//                      (hi.hi, hi.mid, mid.hi, mid.mid, hi.lo, lo.hi), each rotation fragment read from LDS
//                      once for all its pairs.
// Here the token maxima have a row of their own behind T (amax_tok), cleared by the first rotation's first block,
// and the first block of the codes launch writes the scales: no clearing or scaling kernels around the three.
// (Tried and no faster, same box, 4096 and 32768 tokens of 4608 channels: rows of T written in permuted order
// so that the second rotation reads consecutive rows; 16-byte loads of T with a change of layout through
// LDS instead of the 4-byte ones; two accumulator chains instead of four.)
enum DenseSink { kSinkMaxima = 0, kSinkCodes = 1, kSinkRows = 2 };

// eight float32 -> their exact three-way split by truncation, each piece eight bf16 in operand order
// (a byte permute takes the upper halves of two words: no masks for the packing)
__device__ __forceinline__ void split3_bf16(const float (&v)[8], v8bf &hi, v8bf &mid, v8bf &lo)
{
    union { uint32_t u[4]; v8bf v; } h, m, l;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float v0 = v[2 * i], v1 = v[2 * i + 1];
        const uint32_t b0 = __float_as_uint(v0), b1 = __float_as_uint(v1);
        const float r0 = v0 - __uint_as_float(b0 & 0xFFFF0000u), r1 = v1 - __uint_as_float(b1 & 0xFFFF0000u);
        const uint32_t c0 = __float_as_uint(r0), c1 = __float_as_uint(r1);
        const float s0 = r0 - __uint_as_float(c0 & 0xFFFF0000u), s1 = r1 - __uint_as_float(c1 & 0xFFFF0000u);
        h.u[i] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);
        m.u[i] = __builtin_amdgcn_perm(c1, c0, 0x07060302u);
        l.u[i] = __builtin_amdgcn_perm(__float_as_uint(s1), __float_as_uint(s0), 0x07060302u);
    }
    hi = h.v;
    mid = m.v;
    lo = l.v;
}

template <int SINK, int TT, bool GATHER>
__global__ __launch_bounds__(512) void rotate_dense_block_kernel(
    const uint16_t *__restrict__ X, int64_t M, int nb, int64_t ldx, const uint4 *__restrict__ pieces,
    float *__restrict__ amax_tok, float *__restrict__ scale_out, int8_t *__restrict__ Xq,
    const float *__restrict__ Tin, const int32_t *__restrict__ perm, float *__restrict__ Tout, int64_t ldt)
{
    // one token tile of the float32 operand is requested a group ahead (like the bf16 one); two tiles are
    // requested at the top of their own group (no registers to hold both across the products), and the
    // wave that shares the SIMD covers the wait
    constexpr bool AHEAD = GATHER && TT == 1;
    static_assert(!(GATHER && SINK == kSinkRows), "the second rotation ends in maxima or codes");
    constexpr bool QUANT = SINK == kSinkCodes;
    extern __shared__ __align__(16) uint4 lds_pieces[];           // [12][8][64] fragments of this block
    const int K = nb * kBlock;
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    {   // the block's pieces: all twelve requests of a lane in flight, then the LDS writes
        static_assert(kPiecesPerBlock % 512 == 0, "whole rounds of the workgroup");
        constexpr int ROUNDS = kPiecesPerBlock / 512;
        uint4 tmp[ROUNDS];
#pragma unroll
        for (int i = 0; i < ROUNDS; ++i) tmp[i] = pieces[(size_t)b * kPiecesPerBlock + i * 512 + threadIdx.x];
#pragma unroll
        for (int i = 0; i < ROUNDS; ++i) lds_pieces[i * 512 + threadIdx.x] = tmp[i];
    }
    // second rotation: the rows of T that are the block's 128 input channels, and behind them eight waves' worth
    // of rows in which finished codes wait (64 x 8 words per token tile)
    int *const rowtab = reinterpret_cast<int *>(lds_pieces + kPiecesPerBlock);
    uint32_t *const code_lds = reinterpret_cast<uint32_t *>(rowtab + kBlock) + wave * (TT * 8 * 64);
    if constexpr (GATHER) {
        if (threadIdx.x < kBlock) {
            int p = perm[b * kBlock + threadIdx.x];
            rowtab[threadIdx.x] = p < 0 ? 0 : (p >= K ? K - 1 : p);
        }
    }
    __syncthreads();

    constexpr int TOK = 16 * TT;
    const int64_t groups = (M + TOK - 1) / TOK;                   // groups of TT 16-token tiles
    const int64_t stride = (int64_t)gridDim.x * 8;
    // bf16 source: the lane's operand is 16 bytes of its token's row
    auto load_x = [&](v8bf (&xf)[TT][4], int64_t gr) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            int64_t token = gr * TOK + tt * 16 + l16;
            if (token >= M) token = M - 1;                        // repeated rows: their results are not stored
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                union { uint4 u; v8bf v; } ld;
                ld.u = *reinterpret_cast<const uint4 *>(X + token * ldx + b * kBlock + 32 * s + 8 * g);
                xf[tt][s] = ld.v;
            }
        }
    };
    // float32 source: rows of T (token-padded, so tokens past M read what the first rotation wrote for its
    // repeated rows); element e of k-step s is row rowtab[32 s + 8 g + e], token l16 of the tile
    auto gather_x = [&](float (&raw)[4][8], int64_t gr, int tt) {
        const float *const tile = Tin + gr * TOK + tt * 16 + l16;
        int g8 = 8 * g;
        asm volatile("" : "+v"(g8));                              // keeps the row-number reads inside the group loop
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int4 r0 = *reinterpret_cast<const int4 *>(rowtab + 32 * s + g8);
            const int4 r1 = *reinterpret_cast<const int4 *>(rowtab + 32 * s + g8 + 4);
            raw[s][0] = tile[(int64_t)r0.x * ldt]; raw[s][1] = tile[(int64_t)r0.y * ldt];
            raw[s][2] = tile[(int64_t)r0.z * ldt]; raw[s][3] = tile[(int64_t)r0.w * ldt];
            raw[s][4] = tile[(int64_t)r1.x * ldt]; raw[s][5] = tile[(int64_t)r1.y * ldt];
            raw[s][6] = tile[(int64_t)r1.z * ldt]; raw[s][7] = tile[(int64_t)r1.w * ldt];
        }
    };
    auto to_operands = [&](const float (&raw)[4][8], v8bf (&hi)[4], v8bf (&mid)[4], v8bf (&lo)[4]) {
#pragma unroll
        for (int s = 0; s < 4; ++s) split3_bf16(raw[s], hi[s], mid[s], lo[s]);
    };
    int64_t gr = (int64_t)blockIdx.x * 8 + wave;
    v8bf xcur[TT][4], xnext[GATHER ? 1 : TT][4];
    v8bf xmid[GATHER ? TT : 1][4], xlo[GATHER ? TT : 1][4];
    float raw[GATHER ? TT : 1][4][8];
    if (gr < groups) {
        if constexpr (AHEAD) {
            gather_x(raw[0], gr, 0);
            to_operands(raw[0], xcur[0], xmid[0], xlo[0]);
        } else if constexpr (!GATHER) {
            load_x(xcur, gr);
        }
    }
    for (; gr < groups; gr += stride) {
        const int64_t nxt = gr + stride < groups ? gr + stride : gr;  // the last iteration re-reads its own tiles
        if constexpr (AHEAD) {
            gather_x(raw[0], nxt, 0);
        } else if constexpr (GATHER) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) gather_x(raw[tt], gr, tt);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) to_operands(raw[tt], xcur[tt], xmid[tt], xlo[tt]);
        } else {
            load_x(xnext, nxt);
        }
        float inv[TT], amax[TT];
        int64_t token[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            token[tt] = gr * TOK + tt * 16 + l16;
            amax[tt] = 0.0f;
            inv[tt] = 0.0f;
            if constexpr (QUANT) {
                if (token[tt] < M) {
                    const float a = amax_tok[token[tt]];
                    inv[tt] = a > 0.0f ? 127.0f / a : 0.0f;
                    if (scale_out != nullptr && b == 0 && g == 0) scale_out[token[tt]] = a / 127.0f;
                }
            }
        }
        if constexpr (SINK == kSinkRows) {                        // the first block's workgroups clear the maxima
            if (amax_tok != nullptr && b == 0 && lane < TOK) amax_tok[gr * TOK + lane] = 0.0f;
        }
        // the codes of a finished tile wait in registers, or (second rotation, short of registers) in LDS
        uint32_t code[QUANT && !GATHER ? TT : 1][8];
        int lane_off = lane;                                      // keeps the fragment reads inside this loop
        asm volatile("" : "+v"(lane_off));
        // what becomes of a finished tile t (acc[tt][j]: see the sinks above)
        auto finish_tile = [&](int t, const v4f (&acc)[TT]) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                if constexpr (SINK == kSinkCodes) {
                    const uint32_t c = pack4_low_bytes(quant_bits(acc[tt][0], inv[tt]), quant_bits(acc[tt][1], inv[tt]),
                                                       quant_bits(acc[tt][2], inv[tt]), quant_bits(acc[tt][3], inv[tt]));
                    if constexpr (GATHER) code_lds[(tt * 8 + t) * 64 + lane] = c;
                    else code[tt][t] = c;
                } else if constexpr (SINK == kSinkMaxima)
                    amax[tt] = fmaxf(amax[tt], fmaxf(fmaxf(fabsf(acc[tt][0]), fabsf(acc[tt][1])),
                                                     fmaxf(fabsf(acc[tt][2]), fabsf(acc[tt][3]))));
                else                                              // tokens 4 g .. 4 g + 3 of channel c(t, l16)
                    *reinterpret_cast<float4 *>(Tout + (int64_t)(b * kBlock + 32 * (l16 >> 2) + 4 * t + (l16 & 3)) * ldt +
                                                gr * TOK + tt * 16 + 4 * g) =
                        make_float4(acc[tt][0], acc[tt][1], acc[tt][2], acc[tt][3]);
            }
        };
        if constexpr (GATHER) {
            // Fragments in chunks of four (one piece's k-steps of one tile, smallest piece first) through a ring
            // of three: chunk i + 2 is read from LDS while chunk i is multiplied, 4, 8 or 12 instructions
            // (the low piece meets the operand's high piece, the middle one its high and middle, the high one all three).
            uint4 fr[3][4];
            auto request4 = [&](uint4 (&f)[4], int i) {
                const int t = i / 3, p = 2 - i % 3;
#pragma unroll
                for (int s = 0; s < 4; ++s) f[s] = lds_pieces[((p * 4 + s) * 8 + t) * 64 + lane_off];
            };
            request4(fr[0], 0);
            request4(fr[1], 1);
            // Four accumulator chains taken in turn (k-step by k-step, token tile by token tile), so that an
            // instruction never waits for the one before it in its own chain; they are summed when the tile is done.
            constexpr int NCH = 4 / TT;
            v4f ch[TT][NCH];
#pragma unroll
            for (int i = 0; i < 24; ++i) {
                if (i + 2 < 24) request4(fr[(i + 2) % 3], i + 2);
                __builtin_amdgcn_sched_barrier(0);
                const int p = 2 - i % 3;
                if (i % 3 == 0) {
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                        for (int c = 0; c < NCH; ++c) ch[tt][c] = v4f{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int bp = 2; bp >= 0; --bp) {                 // the operand's piece: low, middle, high
                    if (bp + p > 2) continue;                     // pairs below 2^-24 are left out
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        union { uint4 u; v8bf v; } a;
                        a.u = fr[i % 3][s];
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) {
                            const v8bf x = bp == 2 ? xlo[tt][s] : (bp == 1 ? xmid[tt][s] : xcur[tt][s]);
                            ch[tt][s % NCH] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, x, ch[tt][s % NCH], 0, 0, 0);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                if (i % 3 == 2) {
                    v4f acc[TT];
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) {
                        if constexpr (NCH == 4) acc[tt] = (ch[tt][0] + ch[tt][1]) + (ch[tt][2] + ch[tt][3]);
                        else acc[tt] = ch[tt][0] + ch[tt][1];
                    }
                    finish_tile(i / 3, acc);
                }
            }
        } else {
            // the twelve fragments of tile t + 1 are read from LDS while tile t is multiplied (the scheduling
            // barriers keep the reads ahead of the products; left alone, each read is placed right before its use)
            uint4 fa[2][12];
            auto request = [&](uint4 (&f)[12], int t) {
#pragma unroll
                for (int q = 0; q < 12; ++q) f[q] = lds_pieces[(q * 8 + t) * 64 + lane_off];
            };
            request(fa[0], 0);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                if (t + 1 < 8) request(fa[(t + 1) & 1], t + 1);
                __builtin_amdgcn_sched_barrier(0);
                v4f acc[TT];
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[tt] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 11; q >= 0; --q) {                   // smallest piece first
                    union { uint4 u; v8bf v; } a;
                    a.u = fa[t & 1][q];
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) {
                        if constexpr (SINK == kSinkRows)          // rows = tokens, columns = the tile's channels
                            acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xcur[tt][q & 3], a.v, acc[tt], 0, 0, 0);
                        else
                            acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, xcur[tt][q & 3], acc[tt], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                finish_tile(t, acc);
            }
        }
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            if constexpr (SINK == kSinkCodes) {
                uint32_t c[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    if constexpr (GATHER) c[t] = code_lds[(tt * 8 + t) * 64 + lane];
                    else c[t] = code[tt][t];
                }
                if (token[tt] < M) {
                    uint4 *dst = reinterpret_cast<uint4 *>(Xq + token[tt] * K + b * kBlock + 32 * g);
                    dst[0] = make_uint4(c[0], c[1], c[2], c[3]);
                    dst[1] = make_uint4(c[4], c[5], c[6], c[7]);
                }
            } else if constexpr (SINK == kSinkMaxima) {
                float m = fmaxf(amax[tt], __shfl_xor(amax[tt], 16));
                m = fmaxf(m, __shfl_xor(m, 32));
                if (g == 0 && token[tt] < M)
                    atomicMax(reinterpret_cast<unsigned int *>(amax_tok + token[tt]), __float_as_uint(m));
            }
        }
        if constexpr (AHEAD) {
            to_operands(raw[0], xcur[0], xmid[0], xlo[0]);
        } else if constexpr (!GATHER) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int s = 0; s < 4; ++s) xcur[tt][s] = xnext[tt][s];
        }
    }
}

__global__ void dense_clear_kernel(float *sx, int64_t M)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < M) sx[i] = 0.0f;
}

__global__ void dense_scale_kernel(float *sx, int64_t M)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < M) sx[i] = sx[i] / 127.0f;
}

// workgroups along the token axis for the block-resident kernels: as many as fit one round of compute units
int dense_block_chunks(int64_t groups, int nb)
{
    int64_t chunks = num_cus() / nb;            // rounded down: one workgroup more than compute units would wait for a second round
    const int64_t most = (groups + 7) / 8;
    if (chunks > most) chunks = most;
    return chunks < 1 ? 1 : (int)chunks;
}

template <int SINK, int TT, bool GATHER>
hipError_t launch_dense_block_pass(const uint16_t *X, int64_t M, int nb, int64_t ldx, const uint4 *pieces,
                                   float *amax_tok, float *scale_out, int8_t *Xq, const float *Tin, const int32_t *perm, float *Tout, int64_t ldt,
                                   hipStream_t st)
{
    // behind the pieces: the second rotation's 128 row numbers and eight waves' parked codes
    const size_t smem = (size_t)kPiecesPerBlock * 16 + (GATHER ? kBlock * sizeof(int) + 8 * TT * 8 * 64 * sizeof(uint32_t) : 0);
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(rotate_dense_block_kernel<SINK, TT, GATHER>), smem);
        e != hipSuccess)
        return e;
    const int64_t groups = (M + 16 * TT - 1) / (16 * TT);
    hipLaunchKernelGGL((rotate_dense_block_kernel<SINK, TT, GATHER>), dim3((unsigned)dense_block_chunks(groups, nb), nb),
                       dim3(512), smem, st, X, M, nb, ldx, pieces, amax_tok, scale_out, Xq, Tin, perm, Tout, ldt);
    return hipGetLastError();
}

template <int TT>
hipError_t launch_dense_blocks(const uint16_t *X, int64_t M, int nb, int64_t ldx, const uint4 *pieces,
                               int8_t *Xq, float *sx, hipStream_t st)
{
    const unsigned mg = (unsigned)((M + 255) / 256);
    hipLaunchKernelGGL(dense_clear_kernel, dim3(mg), dim3(256), 0, st, sx, M);
    if (hipError_t e = launch_dense_block_pass<kSinkMaxima, TT, false>(X, M, nb, ldx, pieces, sx, nullptr, Xq, nullptr, nullptr,
                                                                       nullptr, 0, st);
        e != hipSuccess)
        return e;
    if (hipError_t e = launch_dense_block_pass<kSinkCodes, TT, false>(X, M, nb, ldx, pieces, sx, nullptr, Xq, nullptr, nullptr,
                                                                      nullptr, 0, st);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL(dense_scale_kernel, dim3(mg), dim3(256), 0, st, sx, M);
    return hipGetLastError();
}

// ---- Eq. 10 in full with dense blocks: (X . Delta) . BlockDiag(R1) . P . BlockDiag(R2) -----------
// frags32[((b * 8 + t) * 8 + s4) * 64 + lane] = four floats: R_b[4 s + g][c(t, r)] for the k-steps
// s = 4 s4 .. 4 s4 + 3 of v_mfma_f32_16x16x4_f32 (lane = 16 g + r, c(t, r) as for the bf16 pieces):
// the A operand of the SECOND rotation, whose B operand is fp32 (first-rotation results).
__global__ __launch_bounds__(256) void rotation_frags32_kernel(const float *__restrict__ R, float *__restrict__ frags)
{
    const int b = blockIdx.y;
    const int idx = blockIdx.x * 256 + threadIdx.x;     // 0 .. 16383: (t, s4, lane, i)
    const int i = idx & 3, lane = (idx >> 2) & 63, s4 = (idx >> 8) & 7, t = idx >> 11;
    const int r = lane & 15, g = lane >> 4;
    const int k = 4 * (4 * s4 + i) + g;
    const int c = 32 * (r >> 2) + 4 * t + (r & 3);
    frags[(size_t)b * kBlock * kBlock + idx] = R[((size_t)b * kBlock + k) * kBlock + c];
}

// One workgroup (a wave per block, at most 12) per group of 16 tokens.  Stage 1 is the dense
// first rotation (bf16 pieces, as above) into an fp32 row buffer T in LDS; stage 2 gathers
// T[perm[.]] as the B operand of fp32 matrix instructions against the second rotation's
// fragments; then the token maximum, the codes and the stores as in the one-rotation kernel.
__global__ __launch_bounds__(768) void rotate_quant_dense_rpr_kernel(
    const uint16_t *__restrict__ X, int64_t M, int nb, int64_t ldx, const uint4 *__restrict__ pieces1,
    const int32_t *__restrict__ perm, const float4 *__restrict__ frags2, int8_t *__restrict__ Xq, float *__restrict__ sx)
{
    extern __shared__ __align__(16) float lds_f[];
    const int K = nb * kBlock;
    const int LDT = K + 4;
    float *const T = lds_f;                              // [16][K + 4]
    float *const amax_s = lds_f + 16 * LDT;              // [2][nw][16]
    const int nw = blockDim.x >> 6;
    int *const srcs = reinterpret_cast<int *>(amax_s + 2 * nw * 16);     // [nw][128]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int64_t groups = (M + 15) / 16;
    const int b = wave;                                  // nw == nb

    // where the second rotation's inputs sit in a row of T: input channel k of block b is channel perm[b*128 + k]
    for (int k = lane; k < kBlock; k += 64) {
        const int p = perm[b * kBlock + k];
        srcs[b * kBlock + k] = p < 0 ? 0 : (p >= K ? K - 1 : p);
    }
    __builtin_amdgcn_wave_barrier();     // a wave only reads its own entries (LDS serves a wave's requests in order)
    int parity = 0;
    for (int64_t tg = blockIdx.x; tg < groups; tg += gridDim.x) {
        const int64_t tok0 = tg * 16;
        float out[1][8][4];
        float unused[1] = {0.0f};
        rotate_block_dense<1>(X, M, ldx, pieces1, b, tok0, lane, out, unused);
#pragma unroll
        for (int t = 0; t < 8; ++t)
            *reinterpret_cast<float4 *>(T + l16 * LDT + b * kBlock + 32 * g + 4 * t) =
                make_float4(out[0][t][0], out[0][t][1], out[0][t][2], out[0][t][3]);
        __syncthreads();
        float bv[32];
#pragma unroll
        for (int s = 0; s < 32; ++s) bv[s] = T[l16 * LDT + srcs[b * kBlock + 4 * s + g]];      // k-step s: k = 4 s + g
        float amax = 0.0f;
        int lane_off = lane;                 // as in rotate_block_dense: keep the loads inside the group loop
        asm volatile("" : "+v"(lane_off));
        const float4 *fb = frags2 + (size_t)b * (kBlock * kBlock / 4) + lane_off;
        float4 fa2[2][8];
        auto request2 = [&](float4 (&f)[8], int t) {
#pragma unroll
            for (int s4 = 0; s4 < 8; ++s4) f[s4] = fb[(t * 8 + s4) * 64];
        };
        request2(fa2[0], 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (t + 1 < 8) request2(fa2[(t + 1) & 1], t + 1);
            __builtin_amdgcn_sched_barrier(0);
            v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s4 = 0; s4 < 8; ++s4) {
                const float4 a4 = fa2[t & 1][s4];
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, bv[4 * s4 + 0], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, bv[4 * s4 + 1], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, bv[4 * s4 + 2], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, bv[4 * s4 + 3], acc, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                out[0][t][j] = acc[j];
                amax = fmaxf(amax, fabsf(acc[j]));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        float *const am = amax_s + parity * nw * 16;
        amax = fmaxf(amax, __shfl_xor(amax, 16));
        amax = fmaxf(amax, __shfl_xor(amax, 32));
        if (g == 0) am[wave * 16 + l16] = amax;
        __syncthreads();        // also: every wave has read its inputs from T before the next group overwrites it
        parity ^= 1;
        float a = 0.0f;
        for (int w = 0; w < nw; ++w) a = fmaxf(a, am[w * 16 + l16]);
        const int64_t token = tok0 + l16;
        const float inv = a > 0.0f ? 127.0f / a : 0.0f;
        if (token < M) {
            if (wave == 0 && g == 0) sx[token] = a / 127.0f;
            store_codes_dense(out[0], inv, Xq + token * K + b * kBlock + 32 * g);
        }
    }
}

// Rows wider than 12 blocks (up to 36): the once-rotated fp32 rows of 16 tokens no longer fit LDS, so a
// workgroup of 12 waves takes 8 tokens (their rows: 8 x (K + 4) floats, 148 KB at K = 4608) and every wave
// several blocks, one after the other.  The matrix instructions still have 16 token columns: stage 1
// rotates 16 consecutive tokens and keeps the first 8, stage 2 reads row (column mod 8).  A wave cannot hold
// the results of three blocks across the exchange of the token maxima, so stage 2 runs twice: once for the
// maxima, once more for the codes.  The gather indices come straight from `perm` (cached reads).
__global__ __launch_bounds__(768) void rotate_quant_dense_rpr_wide_kernel(
    const uint16_t *__restrict__ X, int64_t M, int nb, int64_t ldx, const uint4 *__restrict__ pieces1,
    const int32_t *__restrict__ perm, const float4 *__restrict__ frags2, int8_t *__restrict__ Xq, float *__restrict__ sx)
{
    extern __shared__ __align__(16) float lds_f[];
    const int K = nb * kBlock;
    const int LDT = K + 4;
    float *const T = lds_f;                              // [8][K + 4]
    float *const amax_s = lds_f + 8 * LDT;               // [2][nw][16]
    const int nw = blockDim.x >> 6;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int row = l16 & 7;
    const int64_t groups = (M + 7) / 8;

    // second rotation of block b on the gathered rows: o[t][j] = channel b*128 + 32 g + 4 t + j of token `row`;
    // returns the lane's largest magnitude
    auto second = [&](int b, float (&o)[8][4]) -> float {
        float bv[32];
#pragma unroll
        for (int s = 0; s < 32; ++s) {                   // k-step s: k = 4 s + g
            int p = perm[b * kBlock + 4 * s + g];
            p = p < 0 ? 0 : (p >= K ? K - 1 : p);
            bv[s] = T[row * LDT + p];
        }
        float amax = 0.0f;
        int lane_off = lane;                             // keeps the fragment loads inside the block loop
        asm volatile("" : "+v"(lane_off));
        const float4 *fb = frags2 + (size_t)b * (kBlock * kBlock / 4) + lane_off;
        float4 fa2[2][8];
        auto request2 = [&](float4 (&f)[8], int t) {
#pragma unroll
            for (int s4 = 0; s4 < 8; ++s4) f[s4] = fb[(t * 8 + s4) * 64];
        };
        request2(fa2[0], 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (t + 1 < 8) request2(fa2[(t + 1) & 1], t + 1);
            __builtin_amdgcn_sched_barrier(0);
            v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s4 = 0; s4 < 8; ++s4) {
                const float4 a4 = fa2[t & 1][s4];
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, bv[4 * s4 + 0], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, bv[4 * s4 + 1], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, bv[4 * s4 + 2], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, bv[4 * s4 + 3], acc, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                o[t][j] = acc[j];
                amax = fmaxf(amax, fabsf(acc[j]));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        return amax;
    };

    int parity = 0;
    for (int64_t tg = blockIdx.x; tg < groups; tg += gridDim.x) {
        const int64_t tok0 = tg * 8;
        for (int b = wave; b < nb; b += nw) {
            float out[1][8][4];
            float unused[1] = {0.0f};
            rotate_block_dense<1>(X, M, ldx, pieces1, b, tok0, lane, out, unused);   // tokens tok0 .. tok0 + 15 (clamped to M - 1)
            if (l16 < 8) {
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    *reinterpret_cast<float4 *>(T + l16 * LDT + b * kBlock + 32 * g + 4 * t) =
                        make_float4(out[0][t][0], out[0][t][1], out[0][t][2], out[0][t][3]);
            }
        }
        __syncthreads();
        float amax = 0.0f;
        for (int b = wave; b < nb; b += nw) {
            float o[8][4];
            amax = fmaxf(amax, second(b, o));
        }
        float *const am = amax_s + parity * nw * 16;
        amax = fmaxf(amax, __shfl_xor(amax, 16));
        amax = fmaxf(amax, __shfl_xor(amax, 32));
        if (g == 0) am[wave * 16 + l16] = amax;
        __syncthreads();
        parity ^= 1;
        float a = 0.0f;
        for (int w = 0; w < nw; ++w) a = fmaxf(a, am[w * 16 + l16]);
        const int64_t token = tok0 + row;
        const float inv = a > 0.0f ? 127.0f / a : 0.0f;
        if (wave == 0 && lane < 8 && token < M) sx[token] = a / 127.0f;
        for (int b = wave; b < nb; b += nw) {
            float o[8][4];
            second(b, o);
            if (l16 < 8 && token < M) store_codes_dense(o, inv, Xq + token * K + b * kBlock + 32 * g);
        }
        __syncthreads();                                 // every wave has read T before the next group overwrites it
    }
}

// mag[k] = max over the tokens of |((X . d) . BlockDiag(R_b))[i][k]| (what the zigzag permutation is dealt
// from when the first rotation is dense).  A wave per (token group, block); the 16 tokens of a lane
// row are reduced with row moves, one lane per row merges with an atomic maximum on the bit patterns.
__global__ __launch_bounds__(256) void channel_absmax_dense_kernel(const uint16_t *__restrict__ X, int64_t M, int nb,
                                                                   int64_t ldx, const uint4 *__restrict__ pieces,
                                                                   float *__restrict__ mag)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int b = blockIdx.y;
    const int64_t groups = (M + 15) / 16;
    float mx[8][4];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) mx[t][j] = 0.0f;
    for (int64_t tg = (int64_t)blockIdx.x * 4 + wave; tg < groups; tg += (int64_t)gridDim.x * 4) {
        float out[1][8][4];
        float unused[1] = {0.0f};
        rotate_block_dense<1>(X, M, ldx, pieces, b, tg * 16, lane, out, unused);   // rows past M repeat the last token
#pragma unroll
        for (int t = 0; t < 8; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) mx[t][j] = fmaxf(mx[t][j], fabsf(out[0][t][j]));
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float m = row16_max(mx[t][j]);
            if (l16 == 0) atomicMax(reinterpret_cast<unsigned int *>(mag + b * kBlock + 32 * g + 4 * t + j), __float_as_uint(m));
        }
}

__global__ void dense_fill_zero_kernel(float *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

template <int TT>
hipError_t launch_dense(const uint16_t *X, int64_t M, int nb, int nw, int64_t ldx, const uint4 *pieces,
                        int8_t *Xq, float *sx, hipStream_t st)
{
    const int64_t groups = (M + 16 * TT - 1) / (16 * TT);
    const int64_t grid = groups < num_cus() ? groups : num_cus();      // persistent: one workgroup per compute unit
    const size_t smem = sizeof(float) * 2 * nw * 16 * TT;
    hipLaunchKernelGGL((rotate_quant_dense_kernel<TT>), dim3((unsigned)grid), dim3(64 * nw), smem, st,
                       X, M, nb, ldx, pieces, Xq, sx);
    return hipGetLastError();
}

}  // namespace

size_t rotation_pieces_bytes(int K) { return (size_t)(K / kBlock) * kPiecesPerBlock * 16; }

hipError_t launch_rotation_pieces(const float *R, const float *diag, int K, void *pieces, hipStream_t st)
{
    hipLaunchKernelGGL(rotation_pieces_kernel, dim3(64, K / kBlock), dim3(256), 0, st, R, diag,
                       static_cast<uint16_t *>(pieces));
    return hipGetLastError();
}

size_t rotation_frags32_bytes(int K) { return (size_t)K * kBlock * sizeof(float); }

hipError_t launch_rotation_frags32(const float *R, int K, void *frags, hipStream_t st)
{
    hipLaunchKernelGGL(rotation_frags32_kernel, dim3(64, K / kBlock), dim3(256), 0, st, R, static_cast<float *>(frags));
    return hipGetLastError();
}

hipError_t launch_channel_absmax_dense(const uint16_t *X, int64_t M, int K, int64_t ldx, const void *pieces,
                                       float *mag, hipStream_t st)
{
    hipLaunchKernelGGL(dense_fill_zero_kernel, dim3((K + 255) / 256), dim3(256), 0, st, mag, K);
    if (M == 0) return hipGetLastError();
    const int nb = K / kBlock;
    const int64_t groups = (M + 15) / 16;
    int64_t chunks = (groups + 3) / 4;
    const int64_t most = (256 * 8 + nb - 1) / nb;       // about eight workgroups per compute unit over all blocks
    if (chunks > most) chunks = most;
    hipLaunchKernelGGL(channel_absmax_dense_kernel, dim3((unsigned)chunks, nb), dim3(256), 0, st, X, M, nb, ldx,
                       static_cast<const uint4 *>(pieces), mag);
    return hipGetLastError();
}

bool rotate_quant_dense_supports(int K) { return K % kBlock == 0 && K / kBlock <= 36; }
bool rotate_quant_dense_rpr_supports(int K) { return K % kBlock == 0 && K / kBlock <= 36; }

// Rows wider than 12 blocks have a second form that goes through a workspace: the once-rotated values,
// float32, channel-major, tokens rounded up to 32 (the first rotation writes whole groups of 32 tokens),
// and behind them one row more for the tokens' maxima.  Narrower rows take it from 16384 tokens on, where
// it is ahead of the 16-token kernel (95 against 110 us at 16384 x 1152, 167 against 213 us at 32768 x 1152;
// 44 against 31 us at 4096 x 1152): that kernel streams both rotations' fragments from L2 for every 16 tokens.
static int64_t dense_ws_ldt(int64_t M) { return (M + 31) / 32 * 32; }

size_t rotate_quant_dense_rpr_workspace_bytes(int64_t M, int K)
{
    if (M <= 0 || (K / kBlock <= 12 && M < 16384)) return 0;
    return ((size_t)K + 1) * (size_t)dense_ws_ldt(M) * sizeof(float);
}

hipError_t launch_rotate_quant_dense_rpr_ws(const uint16_t *X, int64_t M, int K, int64_t ldx, const void *pieces1,
                                            const int32_t *perm, const void *pieces2, int8_t *Xq, float *sx,
                                            float *T, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    const int nb = K / kBlock;
    const int64_t ldt = dense_ws_ldt(M);
    float *const amax_tok = T + (size_t)K * ldt;
    // first rotation (also clears the maxima); second rotation for the maxima; again for the codes and the scales
    if (hipError_t e = launch_dense_block_pass<kSinkRows, 2, false>(X, M, nb, ldx, static_cast<const uint4 *>(pieces1),
                                                                    amax_tok, nullptr, Xq, nullptr, nullptr, T, ldt, st);
        e != hipSuccess)
        return e;
    const uint4 *const p2 = static_cast<const uint4 *>(pieces2);
    // Two token tiles per fragment read halve the LDS traffic of the second rotation (4-5 % from 8192 tokens on);
    // with fewer tokens a wave has too few groups of 32 for that to make up for the coarser split of the work.
    if (M >= 8192) {
        if (hipError_t e = launch_dense_block_pass<kSinkMaxima, 2, true>(X, M, nb, ldx, p2, amax_tok, nullptr, Xq, T, perm,
                                                                         nullptr, ldt, st);
            e != hipSuccess)
            return e;
        return launch_dense_block_pass<kSinkCodes, 2, true>(X, M, nb, ldx, p2, amax_tok, sx, Xq, T, perm, nullptr, ldt, st);
    }
    if (hipError_t e = launch_dense_block_pass<kSinkMaxima, 1, true>(X, M, nb, ldx, p2, amax_tok, nullptr, Xq, T, perm,
                                                                     nullptr, ldt, st);
        e != hipSuccess)
        return e;
    return launch_dense_block_pass<kSinkCodes, 1, true>(X, M, nb, ldx, p2, amax_tok, sx, Xq, T, perm, nullptr, ldt, st);
}

hipError_t launch_rotate_quant_dense_rpr(const uint16_t *X, int64_t M, int K, int64_t ldx, const void *pieces1,
                                         const int32_t *perm, const void *frags2, int8_t *Xq, float *sx, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    const int nb = K / kBlock;
    if (nb > 12) {
        // wide rows: 8 tokens per workgroup of 12 waves
        const int64_t groups8 = (M + 7) / 8;
        const int64_t grid8 = groups8 < num_cus() ? groups8 : num_cus();
        const size_t smem8 = sizeof(float) * ((size_t)8 * (K + 4) + 2 * 12 * 16);
        if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(rotate_quant_dense_rpr_wide_kernel), smem8);
            e != hipSuccess)
            return e;
        hipLaunchKernelGGL(rotate_quant_dense_rpr_wide_kernel, dim3((unsigned)grid8), dim3(64 * 12), smem8, st, X, M, nb,
                           ldx, static_cast<const uint4 *>(pieces1), perm, static_cast<const float4 *>(frags2), Xq, sx);
        return hipGetLastError();
    }
    const int64_t groups = (M + 15) / 16;
    const int64_t grid = groups < num_cus() ? groups : num_cus();
    const size_t smem = sizeof(float) * ((size_t)16 * (K + 4) + 2 * nb * 16) + sizeof(int) * (size_t)K;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(rotate_quant_dense_rpr_kernel), smem);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL(rotate_quant_dense_rpr_kernel, dim3((unsigned)grid), dim3(64 * nb), smem, st, X, M, nb, ldx,
                       static_cast<const uint4 *>(pieces1), perm, static_cast<const float4 *>(frags2), Xq, sx);
    return hipGetLastError();
}

hipError_t launch_rotate_quant_dense(const uint16_t *X, int64_t M, int K, int64_t ldx, const void *pieces,
                                     int8_t *Xq, float *sx, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    const int nb = K / kBlock;
    const uint4 *pc = static_cast<const uint4 *>(pieces);
    // Up to 12 blocks: one kernel, a wave per block of a 16-token group (two token tiles per piece load once
    // there are enough tokens to keep every compute unit busy), pieces from L2, activations read once.
    // Wider rows: a workgroup per block with its pieces in LDS, two passes over the activations.
    if (nb <= 12)
        return M >= 8192 ? launch_dense<2>(X, M, nb, nb, ldx, pc, Xq, sx, st) : launch_dense<1>(X, M, nb, nb, ldx, pc, Xq, sx, st);
    return launch_dense_blocks<2>(X, M, nb, ldx, pc, Xq, sx, st);
}

}  // namespace trdq
