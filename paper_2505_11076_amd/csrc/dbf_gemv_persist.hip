// Batch-1 decode as ONE persistent kernel: the matrix-core adder of dbf_gemv_mfma.hip with the
// per-item prologue taken off the critical path.
//
// Timeline measurements of the one-workgroup-per-item kernel show 5-7 us of dependent loads
// (work record -> input vector -> quantise) at the start of every workgroup, at loaded-HBM
// latency, during which that workgroup streams nothing.  Here a workgroup stays resident and
// walks a sequence of items (forward-pass expression of the paper, section 3: B-stage items
// t = ((x . b) B^T) . m, then A-stage items y = (t A^T) . a).  While it streams the sign bits of
// item n it already
//   * holds the record of item n+1,
//   * has the input vector and the row scales of item n+1 in flight into LDS,
//   * lets its tile-prefetch ring run on into the first tiles of item n+1,
// and between two items only compute remains: quantise the staged input into the operand rows.
//
// Asynchronous loads.  The sign tiles go to registers through inline-assembly buffer loads (a
// ring of PF slots per wavefront, waited for with s_waitcnt vmcnt(PF-1)).  Everything else that
// is fetched ahead of time (next input vector, next row scales, the dependency poll) is loaded
// straight into LDS (global_load_lds_*: lane i of the wavefront writes LDS address M0 + size*i,
// inactive lanes write nothing, completion counts in vmcnt), so that no register holds a value
// that is still in flight outside the ring.  The memory pipeline completes a wavefront's loads
// in issue order, and every such load is followed by at least PF ring loads before its first
// use, so the ring's own waits cover it; where no ring loads follow, the wavefront drains.
//
// Items are assigned statically: workgroup g takes items g, g + G, g + 2G, ... of the list (all
// B items first, then all A items; G = workgroups in the launch).  An A item polls its layer's
// "B rows done" counter ahead of time and only in the rare case that the rows are still missing
// at the item boundary does it wait (bounded).  A B item never waits, and a workgroup's items
// come in list order, so every wait ends as long as all workgroups of the launch are resident
// together, which the launcher ensures by sizing the grid with the occupancy query; should the
// bound be hit the wavefront goes on and raises the sticky time-out counter.  The "rows done"
// counters only ever grow: a launch compares them with (epoch + 1) * rows, and the last
// workgroup to leave bumps the epoch, so nothing is reset by the host and a captured launch can
// be replayed.
#include <cstddef>

#include "dbf_kernels.h"

#ifndef DBF_PPF
#define DBF_PPF 4
#endif

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int PF = DBF_PPF;            // tiles of sign bits in flight per wavefront
constexpr float QMAX = 32512.f;        // 127*256: largest |q| so that hi and lo fit int8
constexpr int XQ_PAD = 16;             // bytes of padding per operand row
constexpr unsigned OOB = 0x80000000u;  // buffer offset out of range for any span
constexpr int SPIN_LIMIT = 1 << 18;

__device__ inline float half_bits_to_float(unsigned h) {
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}
__device__ inline uint16_t float_to_half_bits(float f) {
    return __builtin_bit_cast(uint16_t, (_Float16)f);
}
// Wavefront reductions with data-parallel-primitive moves (register to register, a few cycles
// each) instead of LDS-crossbar shuffles (~100 cycles each, six in a chain): butterflies inside
// every row of 16 lanes, then the four row results through scalar registers.
template <int CTRL>
__device__ inline int dpp_move(int v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
__device__ inline float wave_max(float v) {
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<0xB1>(__builtin_bit_cast(int, v))));   // quad_perm [1,0,3,2]
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<0x4E>(__builtin_bit_cast(int, v))));   // quad_perm [2,3,0,1]
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<0x124>(__builtin_bit_cast(int, v))));  // row_ror:4
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<0x128>(__builtin_bit_cast(int, v))));  // row_ror:8
    const int b = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ inline int wave_sum(int v) {
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x124>(v);
    v += dpp_move<0x128>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}

constexpr int REC_DWORDS = (int)(sizeof(DbfItem) / 4);
static_assert(sizeof(DbfItem) % 4 == 0 && REC_DWORDS <= 64, "a record is fetched by one wavefront, one dword per lane");

struct PMisc {
    float scale[2];       // per item parity: u ~= q * scale
    int sigma[2];         // per item parity: sum of q
    float wmax[4];        // per-wavefront max|u| of the input being quantised
    unsigned dep[4];      // per-wavefront landing zone of the dependency poll made during an item
    unsigned poll[4][2];  // per-wavefront early polls: [parity of the polled item's sequence number]
    unsigned rec[4][4][REC_DWORDS];  // per-wavefront ring of prefetched work records
    uint16_t rscale[2][DBF_PERSIST_MAX_SPAN * DBF_TILE_ROWS];  // per item parity: fp16 row scales
};

// LDS-direct loads: lane i of the wavefront stores its 16 (4) bytes at LDS address lds + 16i (4i).
// `lds` must be wavefront-uniform.  M0 is saved and restored around the instruction.
__device__ inline void lds_load16(unsigned lds, const void* p) {
    unsigned save;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(save) : "v"(p), "s"(lds) : "memory");
}
__device__ inline void lds_load16_agent(unsigned lds, const void* p) {
    unsigned save;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off sc1\n\ts_mov_b32 m0, %0"
                 : "=&s"(save) : "v"(p), "s"(lds) : "memory");
}
__device__ inline void lds_load4(unsigned lds, const void* p) {
    unsigned save;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %1, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(save) : "v"(p), "s"(lds) : "memory");
}
__device__ inline void lds_load4_agent(unsigned lds, const void* p) {
    unsigned save;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %1, off sc1\n\ts_mov_b32 m0, %0"
                 : "=&s"(save) : "v"(p), "s"(lds) : "memory");
}
__device__ inline void drain() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// The fields of a work record this kernel uses, read one by one through the scalar cache.
struct PItem {
    const uint8_t* bits;
    const uint16_t* in_scale;
    const uint16_t* row_scale;
    float* t;
    long long io_off;
    int n_ct, nrt, row0, rows, cols, layer, need, stage_a;
};
__device__ inline PItem load_item(const DbfItem* q) {
    PItem r;
    r.bits = q->bits;
    r.in_scale = q->in_scale;
    r.row_scale = q->row_scale;
    r.t = q->t;
    r.io_off = q->io_off;
    r.n_ct = q->n_ct;
    r.nrt = q->nrt;
    r.row0 = q->row0;
    r.rows = q->rows;
    r.cols = q->cols;
    r.layer = q->layer;
    r.need = q->need;
    r.stage_a = q->stage_a;
    return r;
}

// The same from a record that was prefetched into LDS (every value made wavefront-uniform).
__device__ inline PItem item_from_lds(const unsigned* r) {
    auto dw = [&](size_t off) -> unsigned { return (unsigned)__builtin_amdgcn_readfirstlane((int)r[off / 4]); };
    auto qw = [&](size_t off) -> uint64_t { return (uint64_t)dw(off) | ((uint64_t)dw(off + 4) << 32); };
    PItem it;
    it.bits = reinterpret_cast<const uint8_t*>(qw(offsetof(DbfItem, bits)));
    it.in_scale = reinterpret_cast<const uint16_t*>(qw(offsetof(DbfItem, in_scale)));
    it.row_scale = reinterpret_cast<const uint16_t*>(qw(offsetof(DbfItem, row_scale)));
    it.t = reinterpret_cast<float*>(qw(offsetof(DbfItem, t)));
    it.io_off = (long long)qw(offsetof(DbfItem, io_off));
    it.n_ct = (int)dw(offsetof(DbfItem, n_ct));
    it.nrt = (int)dw(offsetof(DbfItem, nrt));
    it.row0 = (int)dw(offsetof(DbfItem, row0));
    it.rows = (int)dw(offsetof(DbfItem, rows));
    it.cols = (int)dw(offsetof(DbfItem, cols));
    it.layer = (int)dw(offsetof(DbfItem, layer));
    it.need = (int)dw(offsetof(DbfItem, need));
    it.stage_a = (int)dw(offsetof(DbfItem, stage_a));
    return it;
}

// What the tile cursor needs to know about an item (wave-uniform).
struct Span {
    v4u rsrc;  // buffer descriptor of the item's sign-bit tiles
    int n_ct, nrt, steps;
};
__device__ inline Span span_of(const PItem& it) {
    Span s;
    const uint64_t a = reinterpret_cast<uint64_t>(it.bits);
    s.rsrc.x = (unsigned)a;
    s.rsrc.y = (unsigned)(a >> 32) & 0xFFFFu;
    s.rsrc.z = (unsigned)(it.nrt * it.n_ct * DBF_TILE_BYTES);
    s.rsrc.w = 0x00020000u;
    s.n_ct = it.n_ct;
    s.nrt = it.nrt;
    s.steps = (((it.n_ct + 3) >> 2) + PF - 1) / PF * PF;  // tiles per wavefront and row tile, padded
    return s;
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4)))
void dbf_decode_persistent_kernel(const DbfItem* __restrict__ items, int n_items, unsigned* __restrict__ psync,
                                  int* __restrict__ timeouts, int n_layers,
                                  const uint16_t* __restrict__ x_base, uint16_t* __restrict__ y_base,
                                  int chs, int n_wg) {
    // LDS: PMisc | operand rows hi, lo [chs] | staged input raw0, raw1 [chs/4 vectors of 16 B] |
    // reduction buffers [2][128][2]
    extern __shared__ __align__(16) unsigned char smem[];
    PMisc* misc = reinterpret_cast<PMisc*>(smem);
    signed char* xq = reinterpret_cast<signed char*>(smem + sizeof(PMisc));
    unsigned char* raw0 = smem + sizeof(PMisc) + 2 * chs;
    unsigned char* raw1 = raw0 + 2 * chs;
    int* red = reinterpret_cast<int*>(raw1 + 2 * chs);
    const unsigned lds0 = (unsigned)reinterpret_cast<size_t>((__attribute__((address_space(3))) unsigned char*)smem);
    const unsigned lds_raw0 = lds0 + (unsigned)sizeof(PMisc) + 2u * chs, lds_raw1 = lds_raw0 + 2u * chs;

    unsigned* done = psync;                   // [n_layers] B row tiles published, ever growing
    unsigned* exited = psync + n_layers;      // workgroups that have left this launch
    // launches completed so far (stable during a launch)
    const unsigned epoch = __hip_atomic_load(psync + n_layers + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const unsigned lane_off = lane * 16;
    const int rho = tid & 127, e_s = rho >> 4;
    const int xrow = (c & 1) * chs + 16 * g;  // operand row of this lane: columns 0/1 = hi/lo, others alias

    // rows of t an A item needs, as a value of the ever-growing counter (wrap-safe compare)
    auto target_of = [&](const PItem& it) -> unsigned { return (epoch + 1u) * (unsigned)it.need; };
    auto reached = [](unsigned counter, unsigned target) -> bool { return (int)(counter - target) >= 0; };

    // ---- asynchronous input of an item into LDS ------------------------------------------------
    // Vector v (8 columns) is handled by thread v % 256, both when loading and when quantising,
    // so a wavefront only ever reads staged data that it loaded itself.
    //   B stage: raw0[v] = 8 fp16 of x, raw1[v] = 8 fp16 of b;  A stage: raw0[v], raw1[v] = 8 fp32 of t.
    // The row scales go straight to their place: rscale[parity][2*tid .. 2*tid+1].
    auto issue_input = [&](const PItem& it, int parity) {
        const int nvec = it.n_ct * 8, nvec_x = it.cols >> 3;
        const unsigned wave_off = 16u * 64u * w;
        if (it.stage_a) {
            for (int v0 = 0; v0 < nvec; v0 += 256) {
                const int v = v0 + tid;
                if (v < nvec) {
                    lds_load16_agent(lds_raw0 + 16u * v0 + wave_off, it.t + 8 * (size_t)v);
                    lds_load16_agent(lds_raw1 + 16u * v0 + wave_off, it.t + 8 * (size_t)v + 4);
                }
            }
        } else {
            const uint16_t* x = x_base + it.io_off;
            for (int v0 = 0; v0 < nvec; v0 += 256) {
                const int v = v0 + tid;
                if (v < nvec_x) lds_load16(lds_raw0 + 16u * v0 + wave_off, x + 8 * (size_t)v);
                if (v < nvec) lds_load16(lds_raw1 + 16u * v0 + wave_off, it.in_scale + 8 * (size_t)v);
            }
        }
        if (2 * tid < it.nrt * DBF_TILE_ROWS) {
            const unsigned dst = lds0 + (unsigned)offsetof(PMisc, rscale) +
                                 (unsigned)parity * (unsigned)sizeof(misc->rscale[0]) + 256u * w;
            lds_load4(dst, it.row_scale + 2 * tid);
        }
    };
    auto values = [&](const PItem& it, int v, float (&u)[8]) {
        if (it.stage_a) {
            const v4f f0 = *reinterpret_cast<const v4f*>(raw0 + 16 * v);
            const v4f f1 = *reinterpret_cast<const v4f*>(raw1 + 16 * v);
            u[0] = f0.x;  u[1] = f0.y;  u[2] = f0.z;  u[3] = f0.w;
            u[4] = f1.x;  u[5] = f1.y;  u[6] = f1.z;  u[7] = f1.w;
        } else if (v < (it.cols >> 3)) {
            const h8 xv = *reinterpret_cast<const h8*>(raw0 + 16 * v);
            const h8 bv = *reinterpret_cast<const h8*>(raw1 + 16 * v);
            u[0] = (float)xv.s0 * (float)bv.s0;  u[1] = (float)xv.s1 * (float)bv.s1;
            u[2] = (float)xv.s2 * (float)bv.s2;  u[3] = (float)xv.s3 * (float)bv.s3;
            u[4] = (float)xv.s4 * (float)bv.s4;  u[5] = (float)xv.s5 * (float)bv.s5;
            u[6] = (float)xv.s6 * (float)bv.s6;  u[7] = (float)xv.s7 * (float)bv.s7;
        } else {  // beyond x the scale b is zero padding
#pragma unroll
            for (int i = 0; i < 8; ++i) u[i] = 0.f;
        }
    };
    // Quantises the (arrived) staged input of `it` into the operand rows.  Contains two barriers;
    // callers make sure that no wavefront still reads the operand rows of the previous item.
    auto quantise = [&](const PItem& it, int parity) {
        const int nvec = it.n_ct * 8;
        float mx = 0.f;
        for (int v = tid; v < nvec; v += 256) {
            float u[8];
            values(it, v, u);
#pragma unroll
            for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(u[i]));
        }
        mx = wave_max(mx);
        if (lane == 0) misc->wmax[w] = mx;
        if (tid == 0) misc->sigma[parity] = 0;
        __syncthreads();
        mx = fmaxf(fmaxf(misc->wmax[0], misc->wmax[1]), fmaxf(misc->wmax[2], misc->wmax[3]));
        const float inv = mx > 0.f ? QMAX / mx : 0.f;
        if (tid == 0) misc->scale[parity] = mx / QMAX;
        signed char* hi_row = xq;
        signed char* lo_row = xq + chs;
        int local = 0;
        for (int v = tid; v < nvec; v += 256) {
            float u[8];
            values(it, v, u);
            unsigned hi4[2] = {0, 0}, lo4[2] = {0, 0};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float f = rintf(u[i] * inv);
                f = fminf(fmaxf(f, -QMAX), QMAX);
                const int q = (int)f;
                const int lo = ((q + 128) & 255) - 128;
                const int hi = (q - lo) >> 8;
                hi4[i >> 2] |= (unsigned)(hi & 255) << (8 * (i & 3));
                lo4[i >> 2] |= (unsigned)(lo & 255) << (8 * (i & 3));
                local += q;
            }
            *reinterpret_cast<uint2*>(hi_row + v * 8) = make_uint2(hi4[0], hi4[1]);
            *reinterpret_cast<uint2*>(lo_row + v * 8) = make_uint2(lo4[0], lo4[1]);
        }
        local = wave_sum(local);
        if (lane == 0) atomicAdd(&misc->sigma[parity], local);
        __syncthreads();
    };
    // Bounded wait until the B rows an A item needs are published (blocking; rare path).
    auto wait_dependency = [&](const PItem& it) {
        const unsigned target = target_of(it);
        int spins = 0;
        while (!reached(__hip_atomic_load(&done[it.layer], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), target)) {
            __builtin_amdgcn_s_sleep(16);
            if (++spins > SPIN_LIMIT) {
                if (lane == 0) __hip_atomic_fetch_add(timeouts, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
        }
    };
    auto poll_dependency = [&](const PItem& it) {
        if (lane == 0) lds_load4_agent(lds0 + (unsigned)offsetof(PMisc, dep) + 4u * w, &done[it.layer]);
    };
    // Look-ahead of a wavefront, by sequence number q of the items its workgroup walks: the record
    // of item q is fetched into slot q % 4 three items ahead, and the dependency of an A item q is
    // polled into poll slot q % 2 two items ahead, so that when q becomes the next item both its
    // record and (normally) the news that its B rows exist are already in LDS.
    auto fetch_record = [&](int q, int idx) {
        if (lane < REC_DWORDS)
            lds_load4(lds0 + (unsigned)offsetof(PMisc, rec) + (unsigned)((w * 4 + (q & 3)) * REC_DWORDS * 4),
                      reinterpret_cast<const unsigned*>(items + idx) + lane);
    };
    auto poll_early = [&](int q, int layer) {
        if (lane == 0)
            lds_load4_agent(lds0 + (unsigned)offsetof(PMisc, poll) + (unsigned)((w * 2 + (q & 1)) * 4), &done[layer]);
    };

    // ---- first item: its prologue is the only exposed one --------------------------------------
    int cur_idx = blockIdx.x;  // the launcher guarantees gridDim.x == n_wg <= n_items
    PItem cur = load_item(items + cur_idx);
    const Span cs = span_of(cur);

    // Tile cursor of the prefetch ring.  It runs PF steps ahead of the step being processed.
    // f_where: 0 = inside the current item, 1 = inside the next item, 2 = at the end of the next
    // item (the record of the one after it is read when the next item becomes current), 3 = no
    // more items.  In states 2 and 3 a fetch is an empty (out-of-range) load; no step is ever
    // processed from such a slot, because every item has at least PF steps.
    v4u f_rsrc = cs.rsrc;
    int f_nct = cs.n_ct, f_nrt = cs.nrt, f_steps = cs.steps;
    int f_rt = 0, f_i = 0, f_where = 0;
    v4u n_rsrc = cs.rsrc;  // the next item as the cursor needs it
    int n_nct = 0, n_nrt = 0, n_steps = PF;
    bool n_known = false, n_valid = false;

    v4u buf[PF];
    auto enter_next = [&]() {
        if (!n_known) {
            f_where = 2;
        } else if (n_valid) {
            f_where = 1;
            f_rsrc = n_rsrc;
            f_nct = n_nct;
            f_nrt = n_nrt;
            f_steps = n_steps;
            f_rt = 0;
            f_i = 0;
        } else {
            f_where = 3;
        }
    };
    auto fetch = [&](v4u& dst) {
        const int ct = w + 4 * f_i;
        const int ok = (int)(f_where < 2) & (int)(ct < f_nct);
        const unsigned off = (unsigned)(f_rt * f_nct + ct) * DBF_TILE_BYTES;
        const unsigned voff = lane_off + (ok ? off : OOB);
        asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen nt" : "=v"(dst) : "v"(voff), "s"(f_rsrc) : "memory");
        if (f_where < 2 && ++f_i == f_steps) {
            f_i = 0;
            if (++f_rt == f_nrt) {
                if (f_where == 0) enter_next();
                else f_where = 2;
            }
        }
    };
    auto wait_slot = [](v4u& slot) {
        asm volatile("s_waitcnt vmcnt(%1)" : "+v"(slot) : "n"(PF - 1) : "memory");
    };
#pragma unroll
    for (int j = 0; j < PF; ++j) fetch(buf[j]);  // in flight during the first prologue

    for (int i = tid; i < 2 * DBF_TILE_ROWS * 2; i += 256) red[i] = 0;
    if (cur.stage_a) wait_dependency(cur);
    int par = 0;
    issue_input(cur, par);
    if (cur_idx + n_wg < n_items) fetch_record(1, cur_idx + n_wg);
    if (cur_idx + 2 * n_wg < n_items) fetch_record(2, cur_idx + 2 * n_wg);
    drain();
    quantise(cur, par);

    int tile_no = 0, seq = 0;
    bool early_next = false;  // an early poll for the item after the current one is in LDS
    for (;;) {
        // ---- look ahead: record and input of the next item ---------------------------------------
        const int nxt_idx = cur_idx + n_wg;
        PItem nxt = cur;
        n_valid = nxt_idx < n_items;
        if (n_valid) nxt = item_from_lds(misc->rec[w][(seq + 1) & 3]);
        // two ahead: poll its dependency now; three ahead: fetch its record
        const bool early_now = early_next;
        early_next = false;
        if (nxt_idx + n_wg < n_items) {
            const unsigned* r2 = misc->rec[w][(seq + 2) & 3];
            const int a2 = __builtin_amdgcn_readfirstlane((int)r2[offsetof(DbfItem, stage_a) / 4]);
            const int l2 = __builtin_amdgcn_readfirstlane((int)r2[offsetof(DbfItem, layer) / 4]);
            if (a2) {
                poll_early(seq + 2, l2);
                early_next = true;
            }
        }
        if (nxt_idx + 2 * n_wg < n_items) fetch_record(seq + 3, nxt_idx + 2 * n_wg);
        {
            const Span ns = span_of(nxt);
            n_rsrc = ns.rsrc;
            n_nct = ns.n_ct;
            n_nrt = ns.nrt;
            n_steps = ns.steps;
        }
        n_known = true;
        if (f_where == 2) enter_next();  // the cursor was waiting at an item end for this record
        const unsigned dep_target = target_of(nxt);
        bool input_issued = false;  // per wavefront: each one stages its own share of the input
        if (n_valid) {
            if (nxt.stage_a) {
                if (early_now && reached(misc->poll[w][(seq + 1) & 1], dep_target)) {
                    issue_input(nxt, par ^ 1);  // the early poll found the rows: full overlap
                    input_issued = true;
                } else {
                    poll_dependency(nxt);  // looked at after the first row tile
                }
            } else {
                issue_input(nxt, par ^ 1);
                input_issued = true;
            }
        }

        // ---- stream the row tiles of the current item ---------------------------------------------
        const int nrt = cur.nrt, n_ct = cur.n_ct, steps = (((n_ct + 3) >> 2) + PF - 1) / PF * PF;
        for (int rtl = 0; rtl < nrt; ++rtl) {
            v4i acc[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) acc[s] = (v4i){0, 0, 0, 0};
            const int xo_max = (n_ct - 1) * 64;
            v4i xop, xnext = *reinterpret_cast<const v4i*>(xq + xrow + min(w * 64, xo_max));
            for (int i0 = 0; i0 < steps; i0 += PF) {
#pragma unroll
                for (int j = 0; j < PF; ++j) {
                    const int xo = (w + 4 * (i0 + j + 1)) * 64;
                    xop = xnext;
                    xnext = *reinterpret_cast<const v4i*>(xq + xrow + min(xo, xo_max));
                    wait_slot(buf[j]);
#pragma unroll
                    for (int s = 0; s < 8; ++s) {
                        const uint32_t msk = 0x01010101u << s;
                        v4i a;
                        a.x = (int)(buf[j].x & msk);
                        a.y = (int)(buf[j].y & msk);
                        a.z = (int)(buf[j].z & msk);
                        a.w = (int)(buf[j].w & msk);
                        acc[s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, xop, acc[s], 0, 0, 0);
                    }
                    fetch(buf[j]);
                }
            }
            // After the very last row tile the ring holds PF placeholder loads that nobody will
            // consume; they must land before the compiler may reuse their registers.
            if (!n_valid && rtl + 1 == nrt) {
                drain();
#pragma unroll
                for (int j = 0; j < PF; ++j) asm volatile("" : "+v"(buf[j]));
            }
            // The dependency poll issued before this row tile has landed (PF or more ring loads
            // were waited for since): start the input of an A item as early as its rows exist.
            if (n_valid && !input_issued) {
                const unsigned seen = misc->dep[w];  // re-read after the ring's waits (memory clobbers)
                if (reached(seen, dep_target)) {
                    issue_input(nxt, par ^ 1);
                    input_issued = true;
                    if (rtl + 1 == nrt) drain();  // no ring loads follow the last row tile
                } else if (rtl + 1 < nrt) {
                    poll_dependency(nxt);  // poll again during the next row tile
                }
            }

            // ---- combine the four wavefronts; finish the rows of this tile ---------------------
            int* rb = red + (tile_no & 1) * DBF_TILE_ROWS * 2;
            if (c < 2) {
#pragma unroll
                for (int s = 0; s < 8; ++s)
#pragma unroll
                    for (int i = 0; i < 4; ++i) atomicAdd(&rb[(16 * s + 4 * g + i) * 2 + c], acc[s][i]);
            }
            ++tile_no;
            __syncthreads();
            if (tid < DBF_TILE_ROWS) {
                const int row = cur.row0 + rtl * DBF_TILE_ROWS + rho;
                const float rscale = half_bits_to_float(misc->rscale[par][rtl * DBF_TILE_ROWS + rho]);
                int vh = rb[rho * 2], vl = rb[rho * 2 + 1];
                rb[rho * 2] = 0;
                rb[rho * 2 + 1] = 0;
                if (e_s < 7) {
                    vh >>= e_s;
                    vl >>= e_s;
                } else {
                    vh = -(vh >> 7);
                    vl = -(vl >> 7);
                }
                const int total = 2 * (vh * 256 + vl) - misc->sigma[par];
                const float val = (float)total * misc->scale[par] * rscale;
                if (cur.stage_a) {
                    if (row < cur.rows) (y_base + cur.io_off)[row] = float_to_half_bits(val);
                } else {
                    __hip_atomic_store(reinterpret_cast<unsigned*>(cur.t) + row, __builtin_bit_cast(unsigned, val),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }

        // ---- item boundary -------------------------------------------------------------------------------
        if (!cur.stage_a) {
            // publish the rows of t: the storing wavefronts wait for their write-through stores
            if (tid < DBF_TILE_ROWS) drain();
            __syncthreads();
            if (tid == 0)
                __hip_atomic_fetch_add(&done[cur.layer], (unsigned)cur.nrt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (!n_valid) break;

        if (!input_issued) {  // rare: the layer's B rows were not there yet
            wait_dependency(nxt);
            issue_input(nxt, par ^ 1);
            drain();
        }
        // All wavefronts are past the last row tile's barrier, so nobody reads the operand rows
        // any more; the staged input has landed (issued at least PF ring loads ago, or drained).
        quantise(nxt, par ^ 1);

        // advance: the next item becomes the current one; the cursor is already inside it
        cur = nxt;
        cur_idx = nxt_idx;
        ++seq;
        par ^= 1;
        n_known = false;
        if (f_where == 1) f_where = 0;  // (2: at the end of it, 3: nothing follows -- both stay)
    }

    // ---- the last workgroup to leave bumps the epoch for the next launch ---------------------------
    if (tid == 0) {
        const unsigned left = __hip_atomic_fetch_add(exited, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (left == (unsigned)n_wg - 1u) {
            __hip_atomic_store(exited, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(psync + n_layers + 1, epoch + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace

// Batch-1 decode of items[0..n_items) (B items first, then A items) in one persistent launch.
// Requirements (checked by the caller): every item has nrt <= DBF_PERSIST_MAX_SPAN, 16-byte
// readable inputs (cols % 8 == 0 for B items, x 16-byte aligned) and max_cols <=
// DBF_PERSIST_MAX_COLS.  psync: [n_layers] rows-done counters, workgroups-left counter, epoch;
// zero before the first launch.  max_wg > 0 caps the grid.
hipError_t dbf_launch_persistent(const DbfItem* items, int n_items, unsigned* psync, int* timeouts,
                                 int n_layers, const void* x_base, void* y_base, int max_cols,
                                 int max_wg, hipStream_t stream) {
    if (n_items <= 0) return hipSuccess;
    if (max_cols > DBF_PERSIST_MAX_COLS) return hipErrorInvalidValue;
    const uint16_t* x = static_cast<const uint16_t*>(x_base);
    uint16_t* y = static_cast<uint16_t*>(y_base);
    const int chs = dbf_col_tiles(max_cols) * DBF_TILE_COLS + XQ_PAD;
    const size_t smem = sizeof(PMisc) + 6 * (size_t)chs + 2 * DBF_TILE_ROWS * 2 * sizeof(int);
    // workgroups of this kernel that fit the GPU at once, cached per LDS size
    static size_t cached_smem = ~(size_t)0;
    static int cached_resident = 0;
    if (cached_smem != smem) {
        int per_cu = 0, device = 0, cus = 0;
        if (hipGetDevice(&device) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(dbf_decode_persistent_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, dbf_decode_persistent_kernel, 256, smem) !=
                hipSuccess ||
            per_cu < 1 || cus < 1)
            return hipErrorUnknown;
        cached_resident = per_cu * cus;
        cached_smem = smem;
    }
    int grid = n_items < cached_resident ? n_items : cached_resident;
    if (max_wg > 0 && grid > max_wg) grid = max_wg;
    hipLaunchKernelGGL(dbf_decode_persistent_kernel, dim3(grid), dim3(256), smem, stream, items, n_items, psync,
                       timeouts, n_layers, x, y, chs, grid);
    return hipGetLastError();
}
