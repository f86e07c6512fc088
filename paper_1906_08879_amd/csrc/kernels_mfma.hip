// Matrix-core sweep kernel for gfx950: the message passing of Section 2.2 step 2,
//   a_v = sum_{u in xi(v)} m_u,   s_v <- s_v + g(a_v),   m_v = f(s_v),
// for H in {32, 64, 128} and one or two layers per network.
//
// One workgroup (4 waves) per (graph, direction) walks the graph's levels in chunks of at
// most 10 nodes.  Design points, all specific to CDNA4:
//   * v_mfma_f32_16x16x32_bf16 with the WEIGHTS as the A operand (16 output columns x 32 k)
//     and the node activations as the B operand.  The fp32 activation of a node is split
//     exactly into three bf16 values (hi, mid, lo); the three parts sit in three adjacent B
//     columns, so one MFMA multiplies the weights with all three parts of five nodes and
//     the three result columns are added with DPP row shifts.  This keeps fp32 accuracy at
//     one third of the MFMA count of three separate passes.
//   * The weight fragments of all layers of one direction live in registers for the whole
//     kernel (bf16 weights: 128 VGPRs at H = 128); only activations move through LDS.
//   * Messages of the last two chunks stay in an LDS table; messages from older chunks are
//     prefetched from HBM one chunk ahead into the same table, so the gather on the
//     critical path reads LDS only.  Chunk records, node ids and the residual inputs are
//     prefetched the same way.
//   * Barriers between layers wait on LDS traffic only, so prefetches stay in flight.
#include "internal.h"

namespace pl {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kThreads = 256;
constexpr int CH = kChunkRows, FCAP = kFarCap, RING = kRing;
constexpr int kTileNodes = 5;                 // nodes per 16-column MFMA tile (3 columns each)
constexpr int NT = CH / kTileNodes;           // column tiles per chunk

// Workgroup barrier that waits for LDS traffic only (global prefetches stay outstanding).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int N>
__device__ __forceinline__ float row_shl(float v)   // lane l reads lane l+N of its row of 16
{
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x100 + N, 0xF, 0xF, true));
}

// x = h + m + l exactly (each part a bf16), for finite x away from the subnormal range.
__device__ __forceinline__ void split3(float x, __bf16 &h, __bf16 &m, __bf16 &l)
{
    h = static_cast<__bf16>(x);
    float r = x - static_cast<float>(h);
    m = static_cast<__bf16>(r);
    r -= static_cast<float>(m);
    l = static_cast<__bf16>(r);
}

__device__ __forceinline__ __bf16 split_part(float x, int s)
{
    __bf16 h, m, l;
    split3(x, h, m, l);
    return s == 0 ? h : (s == 1 ? m : l);
}

struct SweepParams {
    GraphView gv;
    const uint4 *wfrag;     // packed A fragments, see pack_sweep_weights()
    const float *bias;      // [2 dir][2 net][L][H]
    float *emb;             // [n_tot, 2H]
    float *msg;             // [2, n_tot, H]
    uint8_t *reach;         // [2, n_tot]
    const int32_t *cur_node;
};

template <int H, int WS, int L>
__global__ __launch_bounds__(kThreads, 2) void k_sweep_mfma(SweepParams P)
{
    constexpr int MT = H / 16, KS = H / 32;
    constexpr int TPW = (MT + 3) / 4;          // output tiles per wave
    constexpr int NL = 2 * L;                  // layers per chunk: g then f
    constexpr int LDA = H + 8;                 // bf16 row stride of the activation buffers
    constexpr int TPR = H / 4;                 // float4 per message row
    constexpr int PFN = (FCAP * TPR + kThreads - 1) / kThreads;

    __shared__ __attribute__((aligned(16))) float msgtab[kMsgSlots * H];
    __shared__ __attribute__((aligned(16))) __bf16 actbuf[2][NT][16][LDA];
    __shared__ uint8_t flagtab[kMsgSlots + 12];
    __shared__ __attribute__((aligned(16))) float bias_lds[NL * H];

    const int b = blockIdx.x >> 1, dir = blockIdx.x & 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;
    const int jrow = col / 3, spart = col - 3 * jrow;      // col 15: jrow = 5 (unused)
    const bool own = (spart == 0) && (jrow < kTileNodes);  // lane that finishes a node's column

    const GraphView &gv = P.gv;
    const SweepPlanView plan = gv.plan[dir];
    const int32_t *__restrict__ order = gv.order[dir];
    float *__restrict__ msg = P.msg + static_cast<size_t>(dir) * gv.n_tot * H;
    uint8_t *__restrict__ reach = P.reach + static_cast<size_t>(dir) * gv.n_tot;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    const int cl = P.cur_node[b];
    const int cur = (cl >= 0 && cl < n_b) ? n0 + cl : -1;
    const int c_begin = plan.ck_off[b], c_end = plan.ck_off[b + 1];

    // ---- weights of this direction into registers
    bf16x8 A[NL][TPW][KS][WS];
#pragma unroll
    for (int n = 0; n < NL; ++n)
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int mt = wave * TPW + t;
            const int mtc = mt < MT ? mt : MT - 1;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int ws = 0; ws < WS; ++ws) {
                    const size_t at =
                        ((((static_cast<size_t>(dir) * NL + n) * MT + mtc) * KS + ks) * WS + ws) * 64 + lane;
                    const uint4 raw = P.wfrag[at];
                    A[n][t][ks][ws] = *reinterpret_cast<const bf16x8 *>(&raw);
                }
        }
    for (int i = tid; i < NL * H; i += kThreads) bias_lds[i] = P.bias[static_cast<size_t>(dir) * NL * H + i];

    for (int i = tid; i < kMsgSlots * H; i += kThreads) msgtab[i] = 0.0f;
    for (int i = tid; i < 2 * NT * 16 * LDA; i += kThreads) (&actbuf[0][0][0][0])[i] = static_cast<__bf16>(0.0f);
    if (tid < kMsgSlots + 12) flagtab[tid] = 0;

    // ---- software pipeline state
    auto clampc = [&](int c) { return c < c_end ? c : c_end - 1; };
    int4 m0 = plan.meta[c_begin];                      // chunk c
    int4 m1 = plan.meta[clampc(c_begin + 1)];          // chunk c + 1
    uint4 ent0[NT];
    int v0[NT];
    int fid1[PFN];
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        const int r = ct * kTileNodes + (jrow < kTileNodes ? jrow : 0);
        ent0[ct] = plan.ent[static_cast<size_t>(c_begin) * CH + r];
        v0[ct] = order[m0.x + (r < m0.y ? r : 0)];
    }
#pragma unroll
    for (int i = 0; i < PFN; ++i) {
        const int f = (tid + i * kThreads) / TPR;
        fid1[i] = (f < FCAP) ? plan.far[static_cast<size_t>(clampc(c_begin + 1)) * FCAP + f] : -1;
    }
    __syncthreads();

    for (int c = c_begin; c < c_end; ++c) {
        const int rows = m0.y;
        const int ntile = rows > kTileNodes ? 2 : 1;
        const bool has_next = c + 1 < c_end;

        // ---- A: issue every load that does not depend on this chunk's arithmetic
        f32x4 res[TPW][NT];                              // residual inputs s_v of this chunk
#pragma unroll
        for (int t = 0; t < TPW; ++t)
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                const int mt = wave * TPW + t;
                const float4 x = *reinterpret_cast<const float4 *>(
                    P.emb + static_cast<size_t>(v0[ct]) * 2 * H + dir * H + (mt < MT ? mt : 0) * 16 + 4 * kg);
                res[t][ct] = f32x4{x.x, x.y, x.z, x.w};
            }
        float4 pf[PFN];
        int pf_flag[PFN];
#pragma unroll
        for (int i = 0; i < PFN; ++i) {
            const int e = tid + i * kThreads;
            const int f = e / TPR, q = e - f * TPR;
            const bool live = has_next && f < m1.z && fid1[i] >= 0;
            const int u = live ? fid1[i] : m0.x;         // any valid row when not live
            pf[i] = *reinterpret_cast<const float4 *>(msg + static_cast<size_t>(u) * H + 4 * q);
            pf_flag[i] = (live && q == 0) ? ((u == cur) | reach[u]) : 0;
        }
        const int4 m2 = plan.meta[clampc(c + 2)];
        uint4 ent1[NT];
        int v1[NT];
        int fid2[PFN];
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            const int r = ct * kTileNodes + (jrow < kTileNodes ? jrow : 0);
            ent1[ct] = plan.ent[static_cast<size_t>(clampc(c + 1)) * CH + r];
            v1[ct] = order[m1.x + (r < m1.y ? r : 0)];
        }
#pragma unroll
        for (int i = 0; i < PFN; ++i) {
            const int f = (tid + i * kThreads) / TPR;
            fid2[i] = (f < FCAP) ? plan.far[static_cast<size_t>(clampc(c + 2)) * FCAP + f] : -1;
        }

        // ---- layers: gather feeds the first one straight from the message table
        f32x4 acc[TPW][NT];
        int my_bit[NT];
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) my_bit[ct] = 0;

#pragma unroll
        for (int n = 0; n < NL; ++n) {
#pragma unroll
            for (int t = 0; t < TPW; ++t)
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) acc[t][ct] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                if (ct >= ntile) break;
                const int r = ct * kTileNodes + jrow;
                const bool live_col = jrow < kTileNodes && r < rows;
                if (n == 0) {
                    // gather: a_v = sum of neighbour messages, taken from the LDS table
                    const uint32_t w0 = ent0[ct].x, w1 = ent0[ct].y, w2 = ent0[ct].z, w3 = ent0[ct].w;
                    const int cnt_raw = w0 & 0xFFFF;
                    const bool direct = live_col && cnt_raw == 0xFFFF;
                    const int cnt = (live_col && !direct) ? cnt_raw : 0;
                    const int slot[kMaxEnt] = {static_cast<int>(w0 >> 16), static_cast<int>(w1 & 0xFFFF),
                                               static_cast<int>(w1 >> 16), static_cast<int>(w2 & 0xFFFF),
                                               static_cast<int>(w2 >> 16), static_cast<int>(w3 & 0xFFFF),
                                               static_cast<int>(w3 >> 16)};
                    int bit = 0;
#pragma unroll
                    for (int e = 0; e < kMaxEnt; ++e)
                        if (e < cnt) bit |= flagtab[slot[e]];
                    const int v = v0[ct];
                    const int d0 = direct ? gv.nbr_ptr[dir][v] : 0;
                    const int d1 = direct ? gv.nbr_ptr[dir][v + 1] : 0;
                    for (int p = d0; p < d1; ++p) {
                        const int u = gv.nbr_idx[dir][p];
                        bit |= (u == cur) | reach[u];
                    }
                    my_bit[ct] = bit;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        float sum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int e = 0; e < kMaxEnt; ++e) {
                            if (e < cnt) {
                                const float4 *src = reinterpret_cast<const float4 *>(
                                    msgtab + slot[e] * H + 32 * ks + 8 * kg);
                                const float4 x0 = src[0], x1 = src[1];
                                sum[0] += x0.x; sum[1] += x0.y; sum[2] += x0.z; sum[3] += x0.w;
                                sum[4] += x1.x; sum[5] += x1.y; sum[6] += x1.z; sum[7] += x1.w;
                            }
                        }
                        for (int p = d0; p < d1; ++p) {    // rows too wide for the chunk record
                            const float4 *src = reinterpret_cast<const float4 *>(
                                msg + static_cast<size_t>(gv.nbr_idx[dir][p]) * H + 32 * ks + 8 * kg);
                            const float4 x0 = src[0], x1 = src[1];
                            sum[0] += x0.x; sum[1] += x0.y; sum[2] += x0.z; sum[3] += x0.w;
                            sum[4] += x1.x; sum[5] += x1.y; sum[6] += x1.z; sum[7] += x1.w;
                        }
                        bf16x8 frag;
#pragma unroll
                        for (int i = 0; i < 8; ++i) frag[i] = split_part(sum[i], spart);
#pragma unroll
                        for (int t = 0; t < TPW; ++t)
#pragma unroll
                            for (int ws = 0; ws < WS; ++ws)
                                acc[t][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                    A[n][t][ks][ws], frag, acc[t][ct], 0, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        const bf16x8 frag = *reinterpret_cast<const bf16x8 *>(
                            &actbuf[(n - 1) & 1][ct][col][32 * ks + 8 * kg]);
#pragma unroll
                        for (int t = 0; t < TPW; ++t)
#pragma unroll
                            for (int ws = 0; ws < WS; ++ws)
                                acc[t][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                    A[n][t][ks][ws], frag, acc[t][ct], 0, 0, 0);
                    }
                }
            }

            // ---- epilogue: add the three part-columns, bias, ReLU, then hand over
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const int mt = wave * TPW + t;
                if (mt >= MT) continue;
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) {
                    if (ct >= ntile) break;
                    const float4 bv = *reinterpret_cast<const float4 *>(bias_lds + n * H + mt * 16 + 4 * kg);
                    const float bias4[4] = {bv.x, bv.y, bv.z, bv.w};
                    f32x4 y;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float a = acc[t][ct][i];
                        y[i] = fmaxf(a + row_shl<1>(a) + row_shl<2>(a) + bias4[i], 0.0f);
                    }
                    const int r = ct * kTileNodes + jrow;
                    if (!(own && r < rows)) continue;
                    const int v = v0[ct];
                    if (n == L - 1) {                    // end of g: residual update of s_v
#pragma unroll
                        for (int i = 0; i < 4; ++i) y[i] += res[t][ct][i];
                        *reinterpret_cast<float4 *>(P.emb + static_cast<size_t>(v) * 2 * H + dir * H +
                                                    mt * 16 + 4 * kg) = float4{y[0], y[1], y[2], y[3]};
                    }
                    if (n == NL - 1) {                   // end of f: the message of v
                        const float4 out{y[0], y[1], y[2], y[3]};
                        *reinterpret_cast<float4 *>(msg + static_cast<size_t>(v) * H + mt * 16 + 4 * kg) = out;
                        *reinterpret_cast<float4 *>(msgtab + ((c - c_begin) % RING * CH + r) * H + mt * 16 +
                                                    4 * kg) = out;
                    } else {
                        bf16x4 ph, pm, pl;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            __bf16 a, b2, c2;
                            split3(y[i], a, b2, c2);
                            ph[i] = a;
                            pm[i] = b2;
                            pl[i] = c2;
                        }
                        __bf16 *dst = &actbuf[n & 1][ct][col][mt * 16 + 4 * kg];
                        *reinterpret_cast<bf16x4 *>(dst) = ph;
                        *reinterpret_cast<bf16x4 *>(dst + LDA) = pm;
                        *reinterpret_cast<bf16x4 *>(dst + 2 * LDA) = pl;
                    }
                }
            }
            if (n == NL - 1) {
                // reachability bits of this chunk's nodes, then the staged far messages
                if (wave == 0 && kg == 0 && own) {
#pragma unroll
                    for (int ct = 0; ct < NT; ++ct) {
                        const int r = ct * kTileNodes + jrow;
                        if (ct < ntile && r < rows) {
                            reach[v0[ct]] = static_cast<uint8_t>(my_bit[ct]);
                            flagtab[(c - c_begin) % RING * CH + r] =
                                static_cast<uint8_t>(my_bit[ct] | (v0[ct] == cur));
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < PFN; ++i) {
                    const int e = tid + i * kThreads;
                    const int f = e / TPR, q = e - f * TPR;
                    if (has_next && f < m1.z) {
                        const int slot = RING * CH + ((c + 1 - c_begin) & 1) * FCAP + f;
                        *reinterpret_cast<float4 *>(msgtab + slot * H + 4 * q) = pf[i];
                        if (q == 0) flagtab[slot] = static_cast<uint8_t>(pf_flag[i]);
                    }
                }
                __syncthreads();     // also makes this chunk's global messages visible
            } else {
                lds_barrier();
            }
        }

        m0 = m1;
        m1 = m2;
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            ent0[ct] = ent1[ct];
            v0[ct] = v1[ct];
        }
#pragma unroll
        for (int i = 0; i < PFN; ++i) fid1[i] = fid2[i];
    }
}

}  // namespace

// Packs the f and g weights of both directions into MFMA A-operand fragments.
// Index: ((((dir * 2L + n) * MT + mt) * KS + ks) * WS + ws) * 64 + lane, n = g layers then f
// layers; lane l holds W[32 ks + 8 (l / 16) + i][16 mt + l % 16], i = 0..7, as bf16 part ws
// of the exact three-way split (ws = 0 only when the weights are bf16 already).
void pack_sweep_weights(const ModelView &mv, const float *blob, int WS, std::vector<uint16_t> *frag,
                        std::vector<float> *bias)
{
    const int H = mv.H, L = mv.L, MT = H / 16, KS = H / 32, NL = 2 * L;
    frag->assign(static_cast<size_t>(2) * NL * MT * KS * WS * 64 * 8, 0);
    bias->assign(static_cast<size_t>(2) * NL * H, 0.0f);
    auto to_bf16 = [](float x) {
        uint32_t u;
        std::memcpy(&u, &x, 4);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return static_cast<uint16_t>(u >> 16);
    };
    auto from_bf16 = [](uint16_t h) {
        uint32_t u = static_cast<uint32_t>(h) << 16;
        float x;
        std::memcpy(&x, &u, 4);
        return x;
    };
    for (int dir = 0; dir < 2; ++dir)
        for (int n = 0; n < NL; ++n) {
            const LayerRef &lr = (n < L) ? mv.g[dir].layer[n] : mv.f[dir].layer[n - L];
            for (int h = 0; h < H; ++h) (*bias)[(static_cast<size_t>(dir) * NL + n) * H + h] = blob[lr.b + h];
            for (int mt = 0; mt < MT; ++mt)
                for (int ks = 0; ks < KS; ++ks)
                    for (int lane = 0; lane < 64; ++lane)
                        for (int i = 0; i < 8; ++i) {
                            const int k = 32 * ks + 8 * (lane / 16) + i, m = 16 * mt + lane % 16;
                            float rest = blob[lr.w + static_cast<size_t>(k) * H + m];
                            for (int ws = 0; ws < WS; ++ws) {
                                const uint16_t part = to_bf16(rest);
                                rest -= from_bf16(part);
                                const size_t at =
                                    (((((static_cast<size_t>(dir) * NL + n) * MT + mt) * KS + ks) * WS + ws) * 64 + lane) * 8 + i;
                                (*frag)[at] = part;
                            }
                        }
        }
}

bool sweep_mfma_supported(int H, int L, int weight_dtype)
{
    if (L < 1 || L > 2) return false;
    if (weight_dtype == PL_WEIGHTS_BF16) return H == 32 || H == 64 || H == 128;
    return H == 32 || H == 64;
}

void launch_sweep_mfma(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                       const ForwardArgs &fa, const uint4 *wfrag, const float *bias, int WS,
                       hipStream_t s)
{
    if (gv.B == 0) return;
    SweepParams P{gv, wfrag, bias, ws.emb, ws.msg, ws.reach, fa.cur_node};
    const dim3 grid(2 * gv.B), block(kThreads);
#define PL_CASE(HH, WW, LL)                                                      \
    if (mv.H == HH && WS == WW && mv.L == LL) {                                  \
        hipLaunchKernelGGL((k_sweep_mfma<HH, WW, LL>), grid, block, 0, s, P);    \
        return;                                                                  \
    }
    PL_CASE(128, 1, 2) PL_CASE(128, 1, 1)
    PL_CASE(64, 1, 2) PL_CASE(64, 1, 1) PL_CASE(64, 3, 2) PL_CASE(64, 3, 1)
    PL_CASE(32, 1, 2) PL_CASE(32, 1, 1) PL_CASE(32, 3, 2) PL_CASE(32, 3, 1)
#undef PL_CASE
}

}  // namespace pl
