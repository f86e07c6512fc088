// Matrix-core sweep kernel for gfx950: the message passing of Section 2.2 step 2,
//   a_v = sum_{u in xi(v)} m_u,   s_v <- s_v + g(a_v),   m_v = f(s_v),
// for H in {32, 64, 128} and one or two layers per network.
//
// One workgroup (one wave per 16 or 32 output columns, at most four waves) per (graph, direction)
// walks the graph's levels in chunks of at most 8 nodes.  Design points, all specific to
// CDNA4:
//   * v_mfma_f32_16x16x32_bf16 with the node activations as the A operand and the WEIGHTS as
//     the B operand.  The fp32 activation of a node is split exactly into three bf16 values
//     (hi, mid, lo) by truncation; the three parts are three ROWS of A (a fourth row is
//     zero), so a 16-row tile holds four nodes and the three partial products of a node land
//     in one lane's accumulator registers, where they are added: fp32 accuracy from the bf16
//     matrix cores without any cross-lane traffic.
//   * The weight fragments of all layers of one direction live in registers for the whole
//     kernel (bf16 weights: 128 VGPRs per wave at H = 128); only activations move through LDS.
//   * Messages of the last two chunks stay in an LDS table; messages from older chunks are
//     prefetched from HBM one chunk ahead into the same table, so the gather on the
//     critical path reads LDS only.  Chunk records, node ids and the residual inputs (kept
//     in bucket order, so a chunk's rows are contiguous) are prefetched the same way.
//   * Barriers order LDS traffic only, so global prefetches stay in flight across them.
//     A message written to HBM in chunk c is only read back from HBM from chunk c + 3 on
//     (nearer consumers use the LDS table); by then the store has retired, because each
//     wave waits once per chunk for a batch of loads that it issued after that store.
//   * The kernel runs a dependent chain (about a thousand chunks of four layers per graph),
//     so it is bound by instruction issue and LDS round trips, not by HBM bandwidth: the
//     per-layer epilogue is about fifteen instructions per tile.
#include "internal.h"

namespace pl {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int CH = kChunkRows, FCAP = kFarCap, RING = kRing;
constexpr int kTileNodes = 4;                 // nodes per 16-row MFMA tile (hi, mid, lo, zero rows)
constexpr int NT = CH / kTileNodes;           // row tiles per chunk

// Workgroup barrier that orders LDS traffic only: global prefetches stay outstanding.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ uint32_t pack_hi16(float lo_word, float hi_word)
{
    return __builtin_amdgcn_perm(__float_as_uint(hi_word), __float_as_uint(lo_word), 0x07060302u);
}

__device__ __forceinline__ float trunc_bf16(float x)
{
    return __uint_as_float(__float_as_uint(x) & 0xFFFF0000u);
}

struct SweepParams {
    GraphView gv;
    const uint4 *wfrag;     // packed weight fragments, see pack_sweep_weights()
    const float *bias;      // [2 dir][2L layers][H]
    float *emb;             // [n_tot, 2H]   output s_v in node order ([td ; bu])
    float *xb;              // [2, n_tot, H] residual input in bucket order, per direction
    float *msg;             // [2, n_tot, H]
    uint8_t *reach;         // [2, n_tot]
    const int32_t *cur_node;
    int write_xb;           // another sweep follows: keep xb current
    // first sweep: the input x_v = relu(W_in^T phi_v + b_in) (Section 2.2 step 1) is computed
    // here from the node's raw features, kept in bucket order, 16 bytes per node
    const float4 *featb;    // [2, n_tot] {run time, output size, is-visited, bits(device | is-current << 16)}
    const float *proj;      // [(F + 1), H]: rows of W_in, then b_in; NULL when the input comes from xb
    int D;
};

// Reads a chunk's meta record through the constant address space, so that the wave-uniform
// record comes in with a scalar load.
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int4 load_uniform(const int4 *p)
{
    const i32x4 r = *reinterpret_cast<const __attribute__((address_space(4))) i32x4 *>(
        reinterpret_cast<uintptr_t>(p));
    return int4{r.x, r.y, r.z, r.w};
}

constexpr int sweep_waves(int H) { return H / 16 > 4 ? 4 : H / 16; }

template <int H, int WS, int L>
__global__ __launch_bounds__(64 * sweep_waves(H), sweep_waves(H) == 8 ? 4 : 2) void k_sweep_mfma(SweepParams P)
{
    constexpr int NW = sweep_waves(H);         // waves; wave w owns output column tiles w * TPW ...
    constexpr int kThreads = 64 * NW;
    constexpr int NTL = H / 16, KS = H / 32;
    constexpr int TPW = NTL / NW;              // output column tiles per wave
    constexpr int NL = 2 * L;                  // layers per chunk: g then f
    constexpr int LDA = H + 8;                 // bf16 row stride of the activation buffers
    constexpr int TPR = H / 4;                 // float4 per row
    constexpr int PFN = (FCAP * TPR + kThreads - 1) / kThreads;   // staged far float4 per thread
    constexpr int IPR = TPR;                   // gather items per row: one per float4
    constexpr int PGN = (CH * IPR + kThreads - 1) / kThreads;     // gather items per thread
    constexpr int LDM = H + 4;                 // float row stride of the message table
    constexpr int NACC = KS > 1 ? 2 : 1;       // independent accumulation chains per tile
    static_assert(NTL % NW == 0, "column tiles must divide over the waves");

    // message table: H floats per row plus a flag column (1.0 if the node is v* or has v* among
    // the nodes it was computed from, i.e. the reachability bit); the last row stays zero
    __shared__ __attribute__((aligned(16))) float msgtab[(kMsgSlots + 1) * LDM];
    __shared__ __attribute__((aligned(16))) float resbuf[2][CH * H];
    __shared__ __attribute__((aligned(16))) __bf16 actbuf[2][NT * 16][LDA];
    __shared__ int vtab[CH];                      // node ids of the chunk's rows
    __shared__ __attribute__((aligned(16))) float proj_lds[(kMaxD + 5) * H];   // W_in rows, then b_in

    const int b = blockIdx.x >> 1, dir = blockIdx.x & 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;    // MFMA result: column col, node kg of a tile

    const GraphView &gv = P.gv;
    const SweepPlanView plan = gv.plan[dir];
    const int32_t *order = gv.order[dir];
    float *msg = P.msg + static_cast<size_t>(dir) * gv.n_tot * H;
    float *xb = P.xb + static_cast<size_t>(dir) * gv.n_tot * H;
    uint8_t *reach = P.reach + static_cast<size_t>(dir) * gv.n_tot;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    const int cl = P.cur_node[b];
    const int cur = (cl >= 0 && cl < n_b) ? n0 + cl : -1;
    const int c_begin = plan.ck_off[b], c_end = plan.ck_off[b + 1];
    // one row past both directions' messages (and one byte past both directions' bits) is
    // never written: the address of dummy loads, relative to this direction's base
    const int spare_row = (2 - dir) * gv.n_tot;

    // ---- weights of this direction into registers (B operand: lane holds column 16 nt + col)
    bf16x8 W[NL][TPW][KS][WS];
    float bias[NL][TPW];
#pragma unroll
    for (int n = 0; n < NL; ++n)
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int nt = wave * TPW + t;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int ws = 0; ws < WS; ++ws) {
                    const size_t at =
                        ((((static_cast<size_t>(dir) * NL + n) * NTL + nt) * KS + ks) * WS + ws) * 64 + lane;
                    const uint4 raw = P.wfrag[at];
                    W[n][t][ks][ws] = *reinterpret_cast<const bf16x8 *>(&raw);
                }
            bias[n][t] = P.bias[(static_cast<size_t>(dir) * NL + n) * H + nt * 16 + col];
        }
    const bool from_feats = P.proj != nullptr;
    const int D = P.D;
    const float4 *featb = P.featb + static_cast<size_t>(dir) * gv.n_tot;
    if (from_feats)
        for (int i = tid; i < (D + 5) * H; i += kThreads) proj_lds[i] = P.proj[i];
    // x_v[4q .. 4q+3] from a node's raw-feature record
    auto project4 = [&](const f32x4 ft, int q) {
        const float4 *w = reinterpret_cast<const float4 *>(proj_lds) + q;
        const int bits = __float_as_int(ft[3]);
        const int dev = bits & 0xFFFF;
        const float4 bb = w[(D + 4) * (H / 4)], w0 = w[0], w1 = w[H / 4], wd = w[(3 + D) * (H / 4)];
        f32x4 o{bb.x, bb.y, bb.z, bb.w};
        o[0] = fmaf(ft[0], w0.x, o[0]); o[1] = fmaf(ft[0], w0.y, o[1]);
        o[2] = fmaf(ft[0], w0.z, o[2]); o[3] = fmaf(ft[0], w0.w, o[3]);
        o[0] = fmaf(ft[1], w1.x, o[0]); o[1] = fmaf(ft[1], w1.y, o[1]);
        o[2] = fmaf(ft[1], w1.z, o[2]); o[3] = fmaf(ft[1], w1.w, o[3]);
        if (dev < D) {
            const float4 wv = w[(2 + dev) * (H / 4)];
            o[0] += wv.x; o[1] += wv.y; o[2] += wv.z; o[3] += wv.w;
        }
        if (bits >> 16) {
            const float4 wc = w[(2 + D) * (H / 4)];
            o[0] += wc.x; o[1] += wc.y; o[2] += wc.z; o[3] += wc.w;
        }
        o[0] = fmaxf(fmaf(ft[2], wd.x, o[0]), 0.0f); o[1] = fmaxf(fmaf(ft[2], wd.y, o[1]), 0.0f);
        o[2] = fmaxf(fmaf(ft[2], wd.z, o[2]), 0.0f); o[3] = fmaxf(fmaf(ft[2], wd.w, o[3]), 0.0f);
        return o;
    };
    for (int i = tid; i < (kMsgSlots + 1) * LDM; i += kThreads) msgtab[i] = 0.0f;
    for (int i = tid; i < 2 * NT * 16 * LDA; i += kThreads) (&actbuf[0][0][0])[i] = static_cast<__bf16>(0.0f);

    // ---- software pipeline state.  m0 describes chunk c, m1 chunk c + 1.  A gather item is
    // (row r, float4 q) of the chunk: item i of this thread is e = tid + i * kThreads.
    auto clampc = [&](int c) { return c < c_end ? c : c_end - 1; };
    int4 m0 = load_uniform(plan.meta + c_begin);
    int4 m1 = load_uniform(plan.meta + clampc(c_begin + 1));
    u32x4 ent0[PGN];         // neighbour record of the item's row, chunk c
    int vg0[PGN];            // node id of the item's row, chunk c
    int fid1[PFN];           // far sources of chunk c + 1
#pragma unroll
    for (int i = 0; i < PGN; ++i) {
        const int e = tid + i * kThreads;
        const int r = e / IPR;
        const int rr = r < m0.y ? r : 0;
        ent0[i] = *reinterpret_cast<const u32x4 *>(plan.ent + static_cast<size_t>(c_begin) * CH + static_cast<uint32_t>(rr));
        vg0[i] = order[m0.x + rr];
    }
#pragma unroll
    for (int i = 0; i < PFN; ++i) {
        const int f = (tid + i * kThreads) / TPR;
        fid1[i] = (f < FCAP) ? plan.far[static_cast<size_t>(clampc(c_begin + 1)) * FCAP + f] : -1;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PGN; ++i) {            // residual inputs of the first chunk
        const int e = tid + i * kThreads;
        const int r = e / IPR, q = e - r * IPR;
        if (r < m0.y) {
            const f32x4 raw = from_feats ? *reinterpret_cast<const f32x4 *>(featb + m0.x + r)
                                         : *reinterpret_cast<const f32x4 *>(xb + static_cast<size_t>(m0.x + r) * H + 4 * q);
            *reinterpret_cast<f32x4 *>(&resbuf[0][r * H + 4 * q]) = from_feats ? project4(raw, q) : raw;
        }
    }
    __syncthreads();

    for (int c = c_begin; c < c_end; ++c) {
        const int rows = m0.y;
        const int ntile = (rows + kTileNodes - 1) / kTileNodes;
        const bool has_next = c + 1 < c_end;
        const int par = (c - c_begin) & 1;

        // ---- gather: a_v = sum of neighbour messages from the LDS table, split into three
        // bf16 parts, written as three A rows of the first layer
        int my_bit[PGN];
        const int cmax = m0.w;                   // most table entries of any row of the chunk
#pragma unroll
        for (int i = 0; i < PGN; ++i) {
            const int e = tid + i * kThreads;
            const int r = e / IPR, q = e - r * IPR;
            my_bit[i] = 0;
            if (r >= rows) continue;
            const uint32_t w0 = ent0[i].x, w1 = ent0[i].y, w2 = ent0[i].z, w3 = ent0[i].w;
            const int cnt_raw = w0 & 0xFFFF;
            const int cnt = cnt_raw == 0xFFFF ? 0 : cnt_raw;
            const int raw[kMaxEnt] = {static_cast<int>(w0 >> 16), static_cast<int>(w1 & 0xFFFF),
                                      static_cast<int>(w1 >> 16), static_cast<int>(w2 & 0xFFFF),
                                      static_cast<int>(w2 >> 16), static_cast<int>(w3 & 0xFFFF),
                                      static_cast<int>(w3 >> 16)};
            float sum[4] = {0.f, 0.f, 0.f, 0.f};
            float flag = 0.0f;                   // sum of the sources' flag column
#pragma unroll
            for (int k = 0; k < kMaxEnt; ++k) {
                if (k < cmax) {                  // uniform bound; short rows read the zero row
                    const int slot = k < cnt ? raw[k] : kMsgSlots;
                    const float4 x = *reinterpret_cast<const float4 *>(msgtab + slot * LDM + 4 * q);
                    sum[0] += x.x; sum[1] += x.y; sum[2] += x.z; sum[3] += x.w;
                    flag += msgtab[slot * LDM + H];
                }
            }
            if (cnt_raw == 0xFFFF) {
                // a row with more neighbours than its record holds: a list of table slots
                // (recent sources) and node ids (sources at least three chunks back)
                const int d0 = static_cast<int>(w0 >> 16) | (static_cast<int>(w1 & 0xFFFF) << 16);
                const int d1 = d0 + (static_cast<int>(w1 >> 16) | (static_cast<int>(w2 & 0xFFFF) << 16));
                for (int p = d0; p < d1; ++p) {
                    const int u = plan.ovf[p];
                    float4 x;
                    if (u < 0) {
                        x = *reinterpret_cast<const float4 *>(msgtab + (-1 - u) * LDM + 4 * q);
                        flag += msgtab[(-1 - u) * LDM + H];
                    } else {
                        x = *reinterpret_cast<const float4 *>(msg + static_cast<uint32_t>(u * H + 4 * q));
                        flag += ((u == cur) | reach[u]) ? 1.0f : 0.0f;
                    }
                    sum[0] += x.x; sum[1] += x.y; sum[2] += x.z; sum[3] += x.w;
                }
            }
            float rs[4], ls[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                rs[k] = sum[k] - trunc_bf16(sum[k]);
                ls[k] = rs[k] - trunc_bf16(rs[k]);
            }
            __bf16 *dst = &actbuf[0][4 * r][4 * q];      // rows 4r, 4r+1, 4r+2 of the chunk's tiles
            *reinterpret_cast<uint2 *>(dst) = uint2{pack_hi16(sum[0], sum[1]), pack_hi16(sum[2], sum[3])};
            *reinterpret_cast<uint2 *>(dst + LDA) = uint2{pack_hi16(rs[0], rs[1]), pack_hi16(rs[2], rs[3])};
            *reinterpret_cast<uint2 *>(dst + 2 * LDA) = uint2{pack_hi16(ls[0], ls[1]), pack_hi16(ls[2], ls[3])};
            my_bit[i] = flag > 0.0f;             // reachability bit of the row's node
            if (q == 0) vtab[r] = vg0[i];
        }
        lds_barrier();

        // Plain vector types on purpose: arrays of the HIP float4 class that are written in one
        // unrolled branch and read in another are not always split into registers.
        f32x4 pf[PFN];           // far messages of chunk c + 1, in flight during the later layers
        int pf_reach[PFN];
        bool pf_cur[PFN];
        f32x4 pr[PGN];           // residual inputs of chunk c + 1
        int vg1[PGN];
        int4 m2 = m1;
        f32x4 acc[TPW][NT][NACC];

#pragma unroll
        for (int n = 0; n < NL; ++n) {
            // ---- rows of A from LDS (activation parts), weights from registers; the k-steps
            // alternate between two accumulators so that the MFMA chains are half as long
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
#pragma unroll
                for (int t = 0; t < TPW; ++t)
#pragma unroll
                    for (int h = 0; h < NACC; ++h) acc[t][ct][h] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (ct >= ntile) continue;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 a =
                        *reinterpret_cast<const bf16x8 *>(&actbuf[n & 1][16 * ct + col][32 * ks + 8 * kg]);
#pragma unroll
                    for (int t = 0; t < TPW; ++t)
#pragma unroll
                        for (int ws = 0; ws < WS; ++ws)
                            acc[t][ct][ks % NACC] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                a, W[n][t][ks][ws], acc[t][ct][ks % NACC], 0, 0, 0);
                }
            }

            // ---- epilogue: lane (col, kg) holds, for node 4 ct + kg and output column
            // 16 nt + col, the three partial products in acc[..][0..2]
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                if (ct >= ntile) continue;
                const int r = ct * kTileNodes + kg;
                if (r >= rows) continue;
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    const int m = (wave * TPW + t) * 16 + col;
                    float y = acc[t][ct][0][0] + acc[t][ct][0][1] + acc[t][ct][0][2];
                    if constexpr (NACC > 1) y += acc[t][ct][1][0] + acc[t][ct][1][1] + acc[t][ct][1][2];
                    y = fmaxf(y + bias[n][t], 0.0f);
                    if (n == L - 1) {                    // end of g: residual update of s_v
                        y += resbuf[par][r * H + m];
                        P.emb[static_cast<uint32_t>(vtab[r] * 2 * H + dir * H + m)] = y;
                        if (P.write_xb) xb[static_cast<uint32_t>((m0.x + r) * H + m)] = y;
                    }
                    if (n == NL - 1) {                   // end of f: the message of v
                        msg[static_cast<uint32_t>(vtab[r] * H + m)] = y;
                        msgtab[(par * CH + r) * LDM + m] = y;
                    } else {
                        const float rr = y - trunc_bf16(y);
                        const float ll = rr - trunc_bf16(rr);
                        unsigned short *dst =
                            reinterpret_cast<unsigned short *>(&actbuf[(n + 1) & 1][4 * r][m]);
                        dst[0] = static_cast<unsigned short>(__float_as_uint(y) >> 16);
                        dst[LDA] = static_cast<unsigned short>(__float_as_uint(rr) >> 16);
                        dst[2 * LDA] = static_cast<unsigned short>(__float_as_uint(ll) >> 16);
                    }
                }
            }

            if (n == NL - 1) {
                // Wait for this wave's prefetch batch whether or not a lane uses it: the stores
                // that preceded it are then complete too (see the note at the prefetch).
#pragma unroll
                for (int i = 0; i < PFN; ++i) asm volatile("" ::"v"(pf[i][0]), "v"(pf_reach[i]));
                // An offset the compiler cannot see through, defined only here: without it the
                // staged LDS stores below are scheduled right behind their loads, which puts
                // the whole HBM latency back on the critical path.
                int late = 0;
                asm volatile("" : "+v"(late));
                // reachability bits of this chunk's nodes, then the staged data of chunk c + 1
#pragma unroll
                for (int i = 0; i < PGN; ++i) {
                    const int e = tid + i * kThreads;
                    const int r = e / IPR, q = e - r * IPR;
                    if (q == 0 && r < rows) {
                        reach[vg0[i]] = static_cast<uint8_t>(my_bit[i]);
                        msgtab[(par * CH + r) * LDM + H] = (my_bit[i] | (vg0[i] == cur)) ? 1.0f : 0.0f;
                    }
                    if (has_next && r < m1.y)
                        *reinterpret_cast<f32x4 *>(&resbuf[par ^ 1][r * H + 4 * q + late]) =
                            from_feats ? project4(pr[i], q) : pr[i];
                }
#pragma unroll
                for (int i = 0; i < PFN; ++i) {
                    const int e = tid + i * kThreads;
                    const int f = e / TPR, q = e - f * TPR;
                    if (has_next && f < m1.z) {
                        const int slot = RING * CH + (par ^ 1) * FCAP + f;
                        *reinterpret_cast<f32x4 *>(msgtab + slot * LDM + 4 * q + late) = pf[i];
                        if (q == 0) msgtab[slot * LDM + H + late] = ((pf_reach[i] != 0) | pf_cur[i]) ? 1.0f : 0.0f;
                    }
                }
                lds_barrier();
            } else if (n == 0) {
                // The loads for the next chunk are issued here, one layer into the chunk.
                // They may read messages that this workgroup stored to HBM at least two
                // chunks ago.  Those stores are complete: vector memory operations of a wave
                // retire in order, and every wave waited for its own previous batch of these
                // loads (issued after those stores) before the last barrier of the previous
                // chunk (see the end-of-chunk stage above).
                lds_barrier();
#pragma unroll
                for (int i = 0; i < PFN; ++i) {
                    const int e = tid + i * kThreads;
                    const int f = e / TPR, q = e - f * TPR;
                    const bool live = has_next && f < m1.z && fid1[i] >= 0;
                    // lanes without a far source read a spare row that is never written, so
                    // that every wave has a load of this batch to wait for
                    const int u = live ? fid1[i] : spare_row;
                    pf[i] = *reinterpret_cast<const f32x4 *>(msg + static_cast<uint32_t>(u * H + 4 * q));
                    pf_reach[i] = reach[static_cast<uint32_t>(u)];   // combined with pf_cur at the end of the chunk
                    pf_cur[i] = live && u == cur;
                }
                m2 = load_uniform(plan.meta + clampc(c + 2));
#pragma unroll
                for (int i = 0; i < PGN; ++i) {
                    const int e = tid + i * kThreads;
                    const int r = e / IPR, q = e - r * IPR;
                    const int rr = (r < m1.y) ? r : 0;
                    pr[i] = from_feats ? *reinterpret_cast<const f32x4 *>(featb + m1.x + static_cast<uint32_t>(rr))
                                       : *reinterpret_cast<const f32x4 *>(xb + static_cast<size_t>(m1.x) * H +
                                                                          static_cast<uint32_t>(rr * H + 4 * q));
                    ent0[i] = *reinterpret_cast<const u32x4 *>(plan.ent + static_cast<size_t>(clampc(c + 1)) * CH +
                                                              static_cast<uint32_t>(rr));
                    vg1[i] = (order + m1.x)[static_cast<uint32_t>(rr)];
                }
#pragma unroll
                for (int i = 0; i < PFN; ++i) {     // ids staged two chunks ahead of their data
                    const int f = (tid + i * kThreads) / TPR;
                    fid1[i] = (f < FCAP) ? (plan.far + static_cast<size_t>(clampc(c + 2)) * FCAP)[static_cast<uint32_t>(f)] : -1;
                }
            } else {
                lds_barrier();
            }
        }

        m0 = m1;
        m1 = m2;
#pragma unroll
        for (int i = 0; i < PGN; ++i) vg0[i] = vg1[i];
    }
}

// Raw features of every node in the bucket order of both directions (Section 2.1 features;
// the device and the is-current flag travel as bits).
__global__ __launch_bounds__(256) void k_bucket_feats(GraphView gv, const float *__restrict__ feats,
                                                      const int32_t *__restrict__ placement,
                                                      const int32_t *__restrict__ cur_node, int D,
                                                      float4 *__restrict__ featb)
{
    const int v = blockIdx.x * 256 + threadIdx.x;
    if (v >= gv.n_tot) return;
    const int b = gv.node_graph[v];
    const int dev = placement[v];
    const int bits = ((dev >= 0 && dev < D) ? dev : 0xFFFF) | ((v - gv.node_off[b] == cur_node[b]) ? 0x10000 : 0);
    const float4 rec{feats[v * 3 + 0], feats[v * 3 + 1], feats[v * 3 + 2], __int_as_float(bits)};
    featb[gv.pos[0][v]] = rec;
    featb[static_cast<size_t>(gv.n_tot) + gv.pos[1][v]] = rec;
}

}  // namespace

// Packs the f and g weights of both directions into MFMA B-operand fragments.
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
                       bool first_sweep, bool more_sweeps, hipStream_t s)
{
    if (gv.B == 0) return;
    SweepParams P{gv, wfrag, bias, ws.emb, ws.xb, ws.msg, ws.reach, fa.cur_node, more_sweeps ? 1 : 0,
                  ws.featb, first_sweep ? mv.blob + mv.proj.w : nullptr, mv.D};
    if (first_sweep)
        hipLaunchKernelGGL(k_bucket_feats, dim3((gv.n_tot + 255) / 256), dim3(256), 0, s, gv, fa.node_feats,
                           fa.placement, fa.cur_node, mv.D, ws.featb);
    const dim3 grid(2 * gv.B);
#define PL_CASE(HH, WW, LL)                                                      \
    if (mv.H == HH && WS == WW && mv.L == LL) {                                  \
        hipLaunchKernelGGL((k_sweep_mfma<HH, WW, LL>), grid, dim3(64 * sweep_waves(HH)), 0, s, P); \
        return;                                                                  \
    }
    PL_CASE(128, 1, 2) PL_CASE(128, 1, 1)
    PL_CASE(64, 1, 2) PL_CASE(64, 1, 1) PL_CASE(64, 3, 2) PL_CASE(64, 3, 1)
    PL_CASE(32, 1, 2) PL_CASE(32, 1, 1) PL_CASE(32, 3, 2) PL_CASE(32, 3, 1)
#undef PL_CASE
}

}  // namespace pl
