// Run-time simulator of a placement (Appendix, "Simulator"): per device a FIFO queue of
// runnable operations and a FIFO queue of output tensors waiting to leave the device; a device
// runs one operation at a time, its bus carries one tensor at a time, transfers overlap with
// compute; an event loop over op-done and transfer-done events; the run time is the timestamp
// of the last op-done event.
//
// A discrete-event simulation is one dependent chain, so a graph gets one wave, and the batch
// of graphs (rollouts) supplies the parallelism: one workgroup of 64 lanes per graph, the whole
// state of the graph in LDS (children lists, placement, costs, pending-input counters, queue
// links, transfer records).  There are at most 2 D events pending (one per device, one per bus): lane d owns the
// queue and the pending event of device d, lane D + d those of bus d, in registers; the next
// event is a wave-wide minimum over (timestamp, creation number), wake-ups of idle devices and
// buses happen in all lanes at once.  Control flow is uniform over the wave.
//
// Timestamps are float32 with one rounding per operation (no fused multiply-add), and events
// are ordered by (timestamp, creation number): the order is the same as that of a scalar
// implementation of the same rules, event by event.
#include "internal.h"

namespace pl {

namespace {

struct SimLds {
    int32_t *cptr;        // [n + 1] children offsets, graph-local
    float *cost;          // [n]
    float *size;          // [n]
    float *tr_dur;        // [e] transfer records: duration = size of the producer's output / bandwidth
    uint16_t *cidx;       // [e] children, graph-local ids, ascending per node
    uint32_t *node;       // [n] device of the node (bits 0-7) | inputs not yet available on that device << 8
    uint16_t *next_op;    // [n] link of the per-device operation queues
    uint16_t *tr_op;      // [e] transfer records: producer
    uint16_t *tr_next;    // [e] link of the per-bus transfer queues
    uint8_t *tr_dst;      // [e] destination device
    uint16_t *tr_child;   // [e] (one transfer per child) the child the transfer is for
};

__device__ __forceinline__ SimLds carve(unsigned char *base, int n_max, int e_max)
{
    SimLds s;
    unsigned char *p = base;
    s.cptr = reinterpret_cast<int32_t *>(p);   p += sizeof(int32_t) * (n_max + 1);
    s.cost = reinterpret_cast<float *>(p);     p += sizeof(float) * n_max;
    s.size = reinterpret_cast<float *>(p);     p += sizeof(float) * n_max;
    s.tr_dur = reinterpret_cast<float *>(p);   p += sizeof(float) * e_max;
    s.node = reinterpret_cast<uint32_t *>(p);  p += sizeof(uint32_t) * n_max;
    s.cidx = reinterpret_cast<uint16_t *>(p);  p += sizeof(uint16_t) * (e_max + (e_max & 1));
    s.next_op = reinterpret_cast<uint16_t *>(p); p += sizeof(uint16_t) * (n_max + (n_max & 1));
    s.tr_op = reinterpret_cast<uint16_t *>(p); p += sizeof(uint16_t) * (e_max + (e_max & 1));
    s.tr_next = reinterpret_cast<uint16_t *>(p); p += sizeof(uint16_t) * (e_max + (e_max & 1));
    s.tr_dst = p;                                p += e_max + (e_max & 1);
    s.tr_child = reinterpret_cast<uint16_t *>(p);
    return s;
}

constexpr int kNone = 0xFFFF;    // empty link / empty queue

// Minimum of an unsigned value over lanes 0..31 (two DPP rows), returned in every lane.
__device__ __forceinline__ unsigned int row_pair_min(unsigned int v)
{
    const int i0 = static_cast<int>(v);
    unsigned int o;
    o = static_cast<unsigned int>(__builtin_amdgcn_update_dpp(i0, i0, 0xB1, 0xF, 0xF, false));     // quad_perm [1,0,3,2]
    v = o < v ? o : v;
    o = static_cast<unsigned int>(__builtin_amdgcn_update_dpp(static_cast<int>(v), static_cast<int>(v), 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
    v = o < v ? o : v;
    o = static_cast<unsigned int>(__builtin_amdgcn_update_dpp(static_cast<int>(v), static_cast<int>(v), 0x141, 0xF, 0xF, false));  // row_half_mirror
    v = o < v ? o : v;
    o = static_cast<unsigned int>(__builtin_amdgcn_update_dpp(static_cast<int>(v), static_cast<int>(v), 0x140, 0xF, 0xF, false));  // row_mirror
    v = o < v ? o : v;
    const unsigned int r0 = static_cast<unsigned int>(__builtin_amdgcn_readlane(static_cast<int>(v), 0));
    const unsigned int r1 = static_cast<unsigned int>(__builtin_amdgcn_readlane(static_cast<int>(v), 16));
    return r0 < r1 ? r0 : r1;
}

// TL: the timeline is written out as well (for the peak-memory model): start and end of every
// operation, and the time at which an output arrived on every device it was sent to.
// PC: the op-done handler as the appendix prints it: the output is enqueued once for EVERY child
// on another device and a transfer-done event releases that one child (so an output needed by
// several children on one remote device crosses the bus several times; the timeline then keeps
// the first and the last arrival per device).  Otherwise an output crosses once per destination
// device and its arrival releases every child waiting there.
template <bool TL, bool PC>
__global__ __launch_bounds__(64) void k_simulate(GraphView gv, int D, int n_max, int e_max,
                                                 const float *__restrict__ node_feats,
                                                 const int32_t *__restrict__ placement, float inv_bw,
                                                 float *__restrict__ out_runtime,
                                                 int32_t *__restrict__ out_events,
                                                 float *__restrict__ op_start, float *__restrict__ op_end,
                                                 float *__restrict__ arrival, float *__restrict__ arrival_last)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const SimLds S = carve(lds_raw, n_max, e_max);
    const int b = blockIdx.x, lane = threadIdx.x;
    const int n0 = gv.node_off[b], n = gv.node_off[b + 1] - n0;
    const int32_t *gptr = gv.nbr_ptr[1] + n0;            // children CSR (global offsets / ids)
    const int e0 = gptr[0], e = gptr[n] - e0;

    // ---- the graph's state into LDS
    bool bad = false;                                     // a device id outside [0, D)
    for (int v = lane; v < n; v += 64) {
        const int d = placement[n0 + v];
        bad |= d < 0 || d >= D;
        S.cost[v] = node_feats[static_cast<size_t>(n0 + v) * 3 + 0];
        S.size[v] = node_feats[static_cast<size_t>(n0 + v) * 3 + 1];
        S.node[v] = (static_cast<uint32_t>(d) & 0xFFu) |
                    (static_cast<uint32_t>(gv.nbr_ptr[0][n0 + v + 1] - gv.nbr_ptr[0][n0 + v]) << 8);   // number of parents
        S.next_op[v] = kNone;
    }
    for (int v = lane; v <= n; v += 64) S.cptr[v] = gptr[v] - e0;
    for (int i = lane; i < e; i += 64) S.cidx[i] = static_cast<uint16_t>(gv.nbr_idx[1][e0 + i] - n0);
    __syncthreads();
    if (__ballot(bad) != 0ull) {
        if (lane == 0) {
            out_runtime[b] = __builtin_nanf("");
            if (out_events) out_events[b] = -1;
        }
        return;
    }

    // ---- lane-private queue ends and pending event (lane d: device d, lane D + d: bus d)
    int q_head = kNone, q_tail = kNone;
    bool active = false;
    float ev_time = 0.0f;
    int ev_seq = 0, ev_node = 0, ev_dst = 0, ev_child = 0;
    // what the event's handler needs of its operation, read when the event is created (off the
    // handler's chain of dependent LDS reads): its children and the duration of its transfers
    int ev_c0 = 0, ev_cnt = 0;
    float ev_dur = 0.0f;
    int seq = 0, n_tr = 0, n_events = 0;
    float last = 0.0f;

    auto enqueue_op = [&](int dev, int v) {               // uniform arguments
        if (lane == dev) {
            if (q_tail == kNone) q_head = v; else S.next_op[q_tail] = static_cast<uint16_t>(v);
            q_tail = v;
        }
    };
    auto enqueue_transfer = [&](int dev, int o, int dst, float dur, int child) {
        const int k = n_tr++;
        S.tr_op[k] = static_cast<uint16_t>(o);
        S.tr_dst[k] = static_cast<uint8_t>(dst);
        if constexpr (PC) S.tr_child[k] = static_cast<uint16_t>(child);
        S.tr_dur[k] = dur;
        S.tr_next[k] = kNone;
        if (lane == D + dev) {
            if (q_tail == kNone) q_head = k; else S.tr_next[q_tail] = static_cast<uint16_t>(k);
            q_tail = k;
        }
    };
    // idle devices, then idle buses, with a non-empty queue start their next item (the wake-ups)
    auto wake = [&](float now) {
        const bool start = !active && q_head != kNone && lane < 2 * D;
        const unsigned long long m = __ballot(start);
        if (start) {
            const int item = q_head;
            int o, dst = -1, child = 0;
            float dur;
            if (lane < D) {
                o = item;
                q_head = S.next_op[item];
                dur = S.cost[o];
            } else {
                o = S.tr_op[item];
                dst = S.tr_dst[item];
                if constexpr (PC) child = S.tr_child[item];
                q_head = S.tr_next[item];
                dur = S.tr_dur[item];
            }
            ev_child = child;
            if (q_head == kNone) q_tail = kNone;
            active = true;
            ev_c0 = S.cptr[o];
            ev_cnt = S.cptr[o + 1] - ev_c0;
            ev_dur = __fmul_rn(S.size[o], inv_bw);
            ev_time = __fadd_rn(now, dur);
            ev_seq = seq + __popcll(m & ((1ull << lane) - 1ull));
            ev_node = o;
            ev_dst = dst;
            if constexpr (TL) {
                if (lane < D) {
                    op_start[n0 + o] = now;
                    op_end[n0 + o] = ev_time;
                }
            }
        }
        seq += __popcll(m);
    };

    for (int base = 0; base < n; base += 64) {            // operations without parents, ascending id
        const int v = base + lane;
        const uint32_t word = S.node[v < n ? v : 0];
        unsigned long long roots = __ballot(v < n && (word >> 8) == 0);
        while (roots != 0ull) {
            const int l = __ffsll(static_cast<long long>(roots)) - 1;
            roots &= roots - 1;
            enqueue_op(__builtin_amdgcn_readlane(static_cast<int>(word & 0xFFu), l), base + l);
        }
    }
    wake(0.0f);

    const int max_events = n + e + 8;                     // every operation and transfer ends once
    for (int it = 0; it < max_events; ++it) {
        // ---- next event: smallest (timestamp, creation number).  Timestamps are >= 0, so their
        // bit patterns order like the values.  Lanes 0 .. 2 D - 1 (at most two rows of sixteen)
        // hold the candidates: the minimum over each row comes from four DPP steps, the two
        // rows are combined through scalar registers.
        const unsigned int t_bits = active ? __float_as_uint(ev_time) : 0xFFFFFFFFu;
        const unsigned int t_min = row_pair_min(t_bits);
        if (t_min == 0xFFFFFFFFu) break;                  // nothing pending: the simulation is over
        // Usually one pending event carries the smallest timestamp; only ties need the second
        // reduction, over the creation numbers.
        unsigned long long first = __ballot(active && t_bits == t_min);
        if (first & (first - 1)) {
            const unsigned int s_bits = (active && t_bits == t_min) ? static_cast<unsigned int>(ev_seq) : 0xFFFFFFFFu;
            const unsigned int s_min = row_pair_min(s_bits);
            first = __ballot(s_bits == s_min && active && t_bits == t_min);
        }
        const int slot = __ffsll(static_cast<long long>(first)) - 1;
        const float now = __uint_as_float(t_min);
        const int o = __builtin_amdgcn_readlane(ev_node, slot);
        const int dst = __builtin_amdgcn_readlane(ev_dst, slot);
        if (lane == slot) active = false;
        ++n_events;
        // ---- the children of o, one per lane: those on the device where o's output now is
        // (its own device after op-done, the destination after transfer-done) have one input
        // fewer to wait for; after op-done the others make the output cross, once per device.
        // Queues are filled in ascending child id (= lane order), as a scalar loop would.
        const int c0 = __builtin_amdgcn_readlane(ev_c0, slot), cnt = __builtin_amdgcn_readlane(ev_cnt, slot);
        const bool op_done = slot < D;
        const int here = op_done ? slot : dst;
        const float dur = op_done ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ev_dur), slot)) : 0.0f;
        if (op_done) last = now;
        if constexpr (TL) {
            if (!op_done && lane == 0) {
                const size_t at = static_cast<size_t>(n0 + o) * D + dst;
                if constexpr (PC) {
                    if (arrival[at] < 0.0f) arrival[at] = now;       // first crossing to this device
                    arrival_last[at] = now;
                } else {
                    arrival[at] = now;
                }
            }
        }
        if (PC && !op_done) {
            // the transfer was made for one child: it alone has one input fewer to wait for
            const int c = __builtin_amdgcn_readlane(ev_child, slot);
            const uint32_t word = S.node[c];
            if (lane == 0) S.node[c] = word - 0x100u;
            if ((word >> 8) == 1u) enqueue_op(dst, c);
            wake(now);
            continue;
        }
        unsigned int sent = 0;
        for (int base = 0; base < cnt; base += 64) {
            const bool valid = base + lane < cnt;
            const int c = valid ? S.cidx[c0 + base + lane] : 0;
            const uint32_t word = S.node[c];
            const int pc = static_cast<int>(word & 0xFFu);
            const bool same = valid && pc == here;
            const int p = static_cast<int>(word >> 8) - 1;
            if (same) S.node[c] = word - 0x100u;
            unsigned long long ready = __ballot(same && p == 0);
            unsigned long long cross = op_done ? __ballot(valid && pc != here) : 0ull;
            while (ready != 0ull) {
                const int l = __ffsll(static_cast<long long>(ready)) - 1;
                ready &= ready - 1;
                enqueue_op(here, __builtin_amdgcn_readlane(c, l));
            }
            while (cross != 0ull) {
                const int l = __ffsll(static_cast<long long>(cross)) - 1;
                cross &= cross - 1;
                const int pd = __builtin_amdgcn_readlane(pc, l);
                if (PC || ((sent >> pd) & 1u) == 0) {     // once per child, or once per destination
                    sent |= 1u << pd;
                    enqueue_transfer(slot, o, pd, dur, __builtin_amdgcn_readlane(c, l));
                }
            }
        }
        wake(now);
    }
    if (lane == 0) {
        out_runtime[b] = last;
        if (out_events) out_events[b] = n_events;
    }
}

// ---- peak memory of every device from the timeline (appendix "Simulator": the start and end
// timestamps of the operations and the tensor sizes predict the peak memory).  The model: the
// output of v occupies v's device from v's start until the latest of v's end, the end of its last
// consumer there and the arrival of its last outgoing transfer; on another device that consumes
// it, a copy lives from the transfer's arrival until the end of its last consumer there.
// Intervals are half-open [alloc, free).

__global__ __launch_bounds__(256) void k_fill_value(float *__restrict__ p, size_t n, float value)
{
    const size_t idx = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    if (idx < n) p[idx] = value;
}

// One thread per node: alloc[v][d], free[v][d] for every device (-1: no copy there).
__global__ __launch_bounds__(256) void k_lifetimes(GraphView gv, int D, const int32_t *__restrict__ placement,
                                                   const float *__restrict__ op_start,
                                                   const float *__restrict__ op_end,
                                                   const float *__restrict__ arrival,
                                                   const float *__restrict__ arrival_last,
                                                   float *__restrict__ alloc, float *__restrict__ free_t)
{
    // arrival: first crossing to a device (the copy exists from then on); arrival_last: last
    // crossing (the source is kept until then); the same array unless an output may cross twice
    const int v = blockIdx.x * 256 + threadIdx.x;
    if (v >= gv.n_tot) return;
    float *fr = free_t + static_cast<size_t>(v) * D, *al = alloc + static_cast<size_t>(v) * D;
    const int d = placement[v];
    for (int o = 0; o < D; ++o) fr[o] = -1.0f;
    if (d < 0 || d >= D) {                 // the simulator reports the graph as invalid
        for (int o = 0; o < D; ++o) al[o] = -1.0f;
        return;
    }
    // end of the last consumer on every device, kept in this node's own row
    for (int p = gv.nbr_ptr[1][v]; p < gv.nbr_ptr[1][v + 1]; ++p) {
        const int c = gv.nbr_idx[1][p];
        const int pc = placement[c];
        if (pc >= 0 && pc < D) fr[pc] = fmaxf(fr[pc], op_end[c]);
    }
    float own_free = fmaxf(op_end[v], fr[d]);
    for (int o = 0; o < D; ++o) {
        if (o == d) continue;
        const float arr = arrival[static_cast<size_t>(v) * D + o];
        if (arr >= 0.0f) {
            own_free = fmaxf(own_free, arrival_last[static_cast<size_t>(v) * D + o]);   // the source stays until it has been sent
            al[o] = arr;
            fr[o] = fmaxf(arr, fr[o]);
        } else {
            al[o] = -1.0f;
            fr[o] = -1.0f;
        }
    }
    al[d] = op_start[v];
    fr[d] = own_free;
}

// One workgroup per graph: for every device the largest sum of live sizes at any allocation time
// (the sum only grows at an allocation), summed in float64 in ascending node order; then the
// memory-penalised run time R(p) = r if m <= M else r + c (m - M) (appendix, "Reward").
// Per device, the copies that live there are first packed into LDS (alloc, free, size; node order
// kept), padded to a multiple of four with entries that are never live; every packed entry is a
// candidate time, and its live sum runs over the packed entries four at a time.
__global__ __launch_bounds__(256) void k_peak_memory(GraphView gv, int D, int n_max,
                                                     const float *__restrict__ node_feats,
                                                     const float *__restrict__ alloc,
                                                     const float *__restrict__ free_t,
                                                     const float *__restrict__ runtime, float mem_limit,
                                                     float penalty, float *__restrict__ out_peak,
                                                     float *__restrict__ out_reward)
{
    typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int cap = (n_max + 3) / 4 * 4 + 4;
    float *ca = reinterpret_cast<float *>(lds_raw), *cf = ca + cap, *cs = cf + cap;
    __shared__ double red[256];
    __shared__ double peak_all;
    __shared__ int wave_cnt[4];
    __shared__ int packed;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = gv.node_off[b], n = gv.node_off[b + 1] - n0;
    const float r = runtime[b];
    if (!(r == r)) {                       // invalid placement: the simulator wrote NaN
        if (tid == 0 && out_reward) out_reward[b] = r;
        if (out_peak) for (int d = tid; d < D; d += 256) out_peak[static_cast<size_t>(b) * D + d] = r;
        return;
    }
    if (tid == 0) peak_all = 0.0;
    for (int d = 0; d < D; ++d) {
        __syncthreads();
        if (tid == 0) packed = 0;
        __syncthreads();
        for (int base = 0; base < n; base += 256) {
            const int u = base + tid;
            float a = -1.0f, f = -1.0f;
            if (u < n) {
                a = alloc[static_cast<size_t>(n0 + u) * D + d];
                f = free_t[static_cast<size_t>(n0 + u) * D + d];
            }
            const bool have = a >= 0.0f;
            const unsigned long long m = __ballot(have);
            if (lane == 0) wave_cnt[wave] = __popcll(m);
            __syncthreads();
            int pos = packed + __popcll(m & ((1ull << lane) - 1ull));
            for (int w = 0; w < wave; ++w) pos += wave_cnt[w];
            if (have) {
                ca[pos] = a;
                cf[pos] = f;
                cs[pos] = node_feats[static_cast<size_t>(n0 + u) * 3 + 1];
            }
            __syncthreads();
            if (tid == 0) packed += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
            __syncthreads();
        }
        const int k = packed, k4 = (k + 3) / 4 * 4;
        for (int i = k + tid; i < k4; i += 256) {      // padding: allocated after every time, never live
            ca[i] = __builtin_inff();
            cf[i] = -1.0f;
            cs[i] = 0.0f;
        }
        __syncthreads();
        double mx = 0.0;
        for (int i = tid; i < k; i += 256) {
            const float t = ca[i];
            double live = 0.0;
            for (int j = 0; j < k4; j += 4) {
                const f32x4 a4 = *reinterpret_cast<const f32x4 *>(ca + j);
                const f32x4 f4 = *reinterpret_cast<const f32x4 *>(cf + j);
                const f32x4 s4 = *reinterpret_cast<const f32x4 *>(cs + j);
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    live += (a4[q] <= t && t < f4[q]) ? static_cast<double>(s4[q]) : 0.0;
            }
            mx = live > mx ? live : mx;
        }
        red[tid] = mx;
        __syncthreads();
        for (int step = 128; step > 0; step >>= 1) {
            if (tid < step) red[tid] = red[tid + step] > red[tid] ? red[tid + step] : red[tid];
            __syncthreads();
        }
        if (tid == 0) {
            if (out_peak) out_peak[static_cast<size_t>(b) * D + d] = static_cast<float>(red[0]);
            peak_all = red[0] > peak_all ? red[0] : peak_all;
        }
    }
    __syncthreads();
    if (tid == 0 && out_reward) {
        const double m = peak_all, M = static_cast<double>(mem_limit);
        out_reward[b] = m <= M ? r : static_cast<float>(static_cast<double>(r) + static_cast<double>(penalty) * (m - M));
    }
}

}  // namespace

size_t simulator_lds_bytes(int n_max, int e_max)
{
    return sizeof(int32_t) * (n_max + 1) + 2 * sizeof(float) * n_max + sizeof(float) * e_max +
           3 * sizeof(uint16_t) * (e_max + (e_max & 1)) + sizeof(uint32_t) * n_max +
           sizeof(uint16_t) * (n_max + (n_max & 1)) + e_max + 16 + sizeof(uint16_t) * (e_max + 2);
}

int launch_simulate(const GraphView &gv, int D, int n_max, int e_max, const float *node_feats,
                    const int32_t *placement, float inv_bw, bool per_child, float *out_runtime,
                    int32_t *out_events, hipStream_t s)
{
    if (gv.B == 0) return PL_OK;
    const size_t lds = simulator_lds_bytes(n_max, e_max);
    auto run = [&](auto kernel) {
        if (lds > 64 * 1024)
            PL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
        hipLaunchKernelGGL(kernel, dim3(gv.B), dim3(64), lds, s, gv, D, n_max, e_max, node_feats, placement,
                           inv_bw, out_runtime, out_events, nullptr, nullptr, nullptr, nullptr);
        return static_cast<int>(PL_OK);
    };
    return per_child ? run(k_simulate<false, true>) : run(k_simulate<false, false>);
}

// Simulation with the timeline, then lifetimes, peaks and R(p).  scratch: op_start, op_end
// [n_tot]; arrival, arrival_last (used with per_child only), alloc, free_t [n_tot, D].
int launch_simulate_reward(const GraphView &gv, int D, int n_max, int e_max, const float *node_feats,
                           const int32_t *placement, float inv_bw, bool per_child, float mem_limit, float penalty,
                           float *op_start, float *op_end, float *arrival, float *arrival_last, float *alloc,
                           float *free_t, float *runtime, float *out_peak, float *out_reward, int32_t *out_events,
                           hipStream_t s)
{
    if (gv.B == 0) return PL_OK;
    const size_t lds = simulator_lds_bytes(n_max, e_max);
    const size_t nd = static_cast<size_t>(gv.n_tot) * D;
    hipLaunchKernelGGL(k_fill_value, dim3(static_cast<unsigned>((nd + 255) / 256)), dim3(256), 0, s, arrival, nd, -1.0f);
    auto run = [&](auto kernel) {
        if (lds > 64 * 1024)
            PL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
        hipLaunchKernelGGL(kernel, dim3(gv.B), dim3(64), lds, s, gv, D, n_max, e_max, node_feats, placement,
                           inv_bw, runtime, out_events, op_start, op_end, arrival, arrival_last);
        return static_cast<int>(PL_OK);
    };
    const int rc = per_child ? run(k_simulate<true, true>) : run(k_simulate<true, false>);
    if (rc) return rc;
    hipLaunchKernelGGL(k_lifetimes, dim3((gv.n_tot + 255) / 256), dim3(256), 0, s, gv, D, placement, op_start, op_end,
                       arrival, per_child ? arrival_last : arrival, alloc, free_t);
    const size_t lds2 = sizeof(float) * 3 * (static_cast<size_t>(n_max + 3) / 4 * 4 + 4);
    if (lds2 > 48 * 1024)
        PL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(k_peak_memory),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds2)));
    hipLaunchKernelGGL(k_peak_memory, dim3(gv.B), dim3(256), lds2, s, gv, D, n_max, node_feats, alloc, free_t, runtime,
                       mem_limit, penalty, out_peak, out_reward);
    return PL_OK;
}

}  // namespace pl
